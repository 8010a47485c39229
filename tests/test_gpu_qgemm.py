"""rq_qgemm (weight mode) against the oracle: accumulators bit-exact; float outputs within 1e-3;
re-quantized codes equal except at ties."""
import numpy as np
import pytest
import torch

from oracle import repquant_oracle as orc
from tests.helpers import assert_codes_close, assert_float_close, dev, lin_to_device, random_linear

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rq():
    from paper_2402_05628_amd import binding
    return binding, binding.Context(0)


def _act_codes(g, M, K, bits):
    qa = g.integers(0, 2 ** bits, size=(M, K))
    z_a = int(g.integers(0, 2 ** bits))
    return qa, z_a


@pytest.mark.parametrize("M,N,K", [(333, 192, 128), (128, 128, 64), (1000, 768, 768), (2049, 1536, 384), (77, 2304, 768),
                                   (513, 260, 3072)])
@pytest.mark.parametrize("bits_a,bits_w", [(8, 8), (4, 4), (8, 4), (6, 6)])
@pytest.mark.parametrize("tile", [1, 2, 3, 259, 515])      # 259: pipelined, zero-points subtracted in the 4-bit unpack; 515: raw nibbles
def test_accumulators_bit_exact(rq, M, N, K, bits_a, bits_w, tile):
    b, ctx = rq
    print("case", M, N, K, bits_a, bits_w, tile, flush=True)
    b.set_gemm_tile(ctx, tile)
    try:
        g = np.random.default_rng(M + N + K + bits_a)
        qa, z_a = _act_codes(g, M, K, bits_a)
        lin = random_linear(g, N, K, bits_w)
        want = orc.qlinear_acc(qa, z_a, lin["codes"], lin["z_w"])
        a_off = b.store_offset(bits_a, z_a)
        A = dev((qa - a_off).astype(np.int8))
        rs = torch.empty(M, dtype=torch.int32, device="cuda")
        b.rq_rowsum_i8(ctx, A, rs)
        acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
        b.rq_qgemm(ctx, A, a_off, z_a, 0.01, lin_to_device(lin, bits_w), out_acc=acc, rowsum_a=rs)
        torch.cuda.synchronize()
        assert np.array_equal(acc.cpu().numpy().astype(np.int64), want)
    finally:
        b.set_gemm_tile(ctx, 0)


@pytest.mark.parametrize("M,N,K,tile", [(1990, 3072, 256, 7), (1990, 3072, 2048, 7), (2048, 6144, 256, 8), (1000, 4096, 128, 5),
                                        (700, 8192, 192, 6)])
@pytest.mark.parametrize("bits_a,bits_w", [(4, 4), (8, 8)])
def test_accumulators_few_tile_rows_many_tile_columns(rq, M, N, K, tile, bits_a, bits_w):
    """Few tile rows, many tile columns (every XCD's range of the tile list spans many columns; ragged last tile row):
    every output written exactly once: true accumulators, no sentinel left."""
    b, ctx = rq
    print("case", M, N, K, tile, bits_a, bits_w, flush=True)
    b.set_gemm_tile(ctx, tile)
    try:
        g = np.random.default_rng(M + N + K + tile)
        qa, z_a = _act_codes(g, M, K, bits_a)
        lin = random_linear(g, N, K, bits_w)
        want = orc.qlinear_acc(qa, z_a, lin["codes"], lin["z_w"])
        a_off = b.store_offset(bits_a, z_a)
        A = dev((qa - a_off).astype(np.int8))
        rs = torch.empty(M, dtype=torch.int32, device="cuda")
        b.rq_rowsum_i8(ctx, A, rs)
        acc = torch.full((M, N), -(2 ** 31) + 5, dtype=torch.int32, device="cuda")
        b.rq_qgemm(ctx, A, a_off, z_a, 0.01, lin_to_device(lin, bits_w), out_acc=acc, rowsum_a=rs)
        torch.cuda.synchronize()
        assert np.array_equal(acc.cpu().numpy().astype(np.int64), want)
    finally:
        b.set_gemm_tile(ctx, 0)


def test_accumulator_extremes(rq):
    """All-max codes against all-min weights at K = 11008: the largest magnitudes the int32 contract allows."""
    b, ctx = rq
    M, N, K = 130, 128, 11008
    qa = np.full((M, K), 255)
    lin = dict(codes=np.zeros((N, K), np.int64), s_w=np.full(N, 1e-3, np.float32), z_w=np.full(N, 255), bias=None)
    lin["codes"][::2] = 255
    lin["z_w"][::2] = 0
    want = orc.qlinear_acc(qa, 0, lin["codes"], lin["z_w"])
    a_off = b.store_offset(8, 0)
    A = dev((qa - a_off).astype(np.int8))
    rs = torch.empty(M, dtype=torch.int32, device="cuda")
    b.rq_rowsum_i8(ctx, A, rs)
    acc = torch.zeros((M, N), dtype=torch.int32, device="cuda")
    b.rq_qgemm(ctx, A, a_off, 0, 0.01, lin_to_device(lin, 8), out_acc=acc, rowsum_a=rs)
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), want)
    assert np.abs(want).max() == 255 * 255 * K


@pytest.mark.parametrize("bits_a,bits_w", [(8, 8), (4, 4), (8, 4)])
@pytest.mark.parametrize("M,tile", [(515, 0), (515, 4), (963, 4), (320, 4), (515, 5), (192, 5), (770, 5), (515, 8), (770, 8),
                                    (256, 8)])
def test_float_output_bias_residual(rq, bits_a, bits_w, M, tile):
    """tile 4 takes the 320-row tiles (one workgroup per CU) that large single-wave launches use, tile 5 the 192-row
    tiles (two per CU) that launches with a short K loop use, tile 8 the 256 x 256 tiles of large products with packed
    4-bit weights."""
    b, ctx = rq
    N, K = 384, 256
    print("case", bits_a, bits_w, M, tile, flush=True)
    g = np.random.default_rng(11 + bits_a + M)
    qa, z_a = _act_codes(g, M, K, bits_a)
    lin = random_linear(g, N, K, bits_w)
    res = g.normal(size=(M, N)).astype(np.float32) * 3
    s_a = np.float32(0.037)
    want = orc.qlinear(qa, s_a, z_a, lin) + res
    a_off = b.store_offset(bits_a, z_a)
    A = dev((qa - a_off).astype(np.int8))
    rs = torch.empty(M, dtype=torch.int32, device="cuda")
    b.rq_rowsum_i8(ctx, A, rs)
    out = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    b.set_gemm_tile(ctx, tile)
    try:
        b.rq_qgemm(ctx, A, a_off, z_a, float(s_a), lin_to_device(lin, bits_w), residual=dev(res), out_f32=out, rowsum_a=rs)
        torch.cuda.synchronize()
    finally:
        b.set_gemm_tile(ctx, 0)
    assert_float_close(out.cpu().numpy(), want, "qgemm f32")


@pytest.mark.parametrize("bits_a,bits_w,bits_o", [(8, 8, 8), (4, 4, 4), (6, 6, 6), (8, 4, 8)])
@pytest.mark.parametrize("act,tile", [("none3", 0), ("gelu", 0), ("gated", 0), ("gelu_q_only", 0), ("gated_q_only", 0),
                                      ("none3", 5), ("none3", 6), ("none3", 7), ("gelu_q_only", 5), ("gelu_q_only", 6),
                                      ("gated_q_only", 5), ("gated_q_only", 6), ("gated_q_only", 7),
                                      ("none3", 8), ("gelu_q_only", 8), ("gated_q_only", 8),
                                      ("none3", 512), ("none3", 517), ("gelu_q_only", 518), ("gated_q_only", 519), ("none3", 520)])
def test_requantized_output(rq, bits_a, bits_w, bits_o, act, tile):
    """tile 5 / 6 / 7: the 192- / 128- / 256-row tiles of the kernel that writes re-quantized codes only; 8: 256 x 256 tiles;
    + 512: the same with the raw-nibble variant of the packed 4-bit weights at this short K (the row sums are passed either way; by
    default the variant is taken for K >= 2048, as in the large-product and long-K tests below)."""
    b, ctx = rq
    q_only = act.endswith("_q_only")      # the block's launches: re-quantized codes are the only output
    act = act.replace("_q_only", "")
    M, K = 301, 256
    b.set_gemm_tile(ctx, tile)
    try:
        _requantized_output_case(b, ctx, bits_a, bits_w, bits_o, act, q_only, M, K)
    finally:
        b.set_gemm_tile(ctx, 0)


@pytest.mark.parametrize("bits_a,bits_w,bits_o", [(8, 8, 8), (4, 4, 4), (6, 6, 6), (8, 4, 8)])
@pytest.mark.parametrize("act,M,K", [("none3", 520, 1024), ("gelu_q_only", 301, 896), ("gated_q_only", 700, 768), ("none3", 257, 384)])
def test_requantized_output_wide_tiles_long_k(rq, bits_a, bits_w, bits_o, act, M, K):
    """The 256 x 256 tiles with a K loop long enough for the ring to be refilled (in pairs of stages) several times."""
    b, ctx = rq
    q_only = act.endswith("_q_only")
    b.set_gemm_tile(ctx, 8)
    try:
        _requantized_output_case(b, ctx, bits_a, bits_w, bits_o, act.replace("_q_only", ""), q_only, M, K)
    finally:
        b.set_gemm_tile(ctx, 0)


@pytest.mark.timeout(300)
@pytest.mark.parametrize("bits_a,bits_w,bits_o", [(4, 4, 4), (8, 6, 8)])
def test_requantized_output_large_product(rq, bits_a, bits_w, bits_o):
    """A product large enough for the launcher to pick the 256 x 256 tiles by itself and to walk them in bands of several
    tile rows (9 tile rows: the last band is a partial one, and the last tile row is ragged).  Sampled rows of every band
    against the oracle; a sentinel shows that every tile was written."""
    b, ctx = rq
    M, N, K = 2264, 14592, 2048
    g = np.random.default_rng(11 + bits_w)
    qa, z_a = _act_codes(g, M, K, bits_a)
    lin = random_linear(g, N, K, bits_w)
    s_a = np.float32(1.5 / (np.sqrt(K) * (2 ** bits_a / 3.46) * (2 ** bits_w / 3.46) * 3e-3))
    rows = np.concatenate([np.arange(0, 24), np.arange(1000, 1024), np.arange(1530, 1546), np.arange(2040, 2064), np.arange(M - 24, M)])
    y = orc.qlinear(qa[rows], s_a, z_a, lin)
    s_o = np.float32((y.max() - y.min()) / (2 ** bits_o - 1))
    z_o = int(np.rint(-y.min() / np.float64(s_o)))
    want = orc.uniform_quant(y, s_o, z_o, bits_o)
    off_o = b.store_offset(bits_o, z_o)
    a_off = b.store_offset(bits_a, z_a)
    A = dev((qa - a_off).astype(np.int8))
    rs = torch.empty(M, dtype=torch.int32, device="cuda")
    b.rq_rowsum_i8(ctx, A, rs)
    sentinel = 99 if bits_o < 8 else None      # stored codes of fewer than 8 bits lie in [-off, 2^bits - 1 - off], off <= 2^bits - 1
    out = torch.full((M, N), 99, dtype=torch.int8, device="cuda")
    print("case large", bits_a, bits_w, bits_o, flush=True)
    b.rq_qgemm(ctx, A, a_off, z_a, float(s_a), lin_to_device(lin, bits_w), out_q=out, bits_o=bits_o, s_o=[float(s_o)], z_o=[z_o],
               off_o=[off_o], seg_len=N, rowsum_a=rs)
    if sentinel is not None:
        assert not bool((out == sentinel).any()), "some output tile was never written"
    got = out[torch.as_tensor(rows, device="cuda")].cpu().numpy().astype(np.int64) + off_o
    assert_codes_close(got, want, "large product, sampled rows")


def _requantized_output_case(b, ctx, bits_a, bits_w, bits_o, act, q_only, M, K):
    N = 384 if act != "gated" else 512
    g = np.random.default_rng(5 + bits_a + len(act))
    qa, z_a = _act_codes(g, M, K, bits_a)
    lin = random_linear(g, N, K, bits_w)
    s_a = np.float32(1.5 / (np.sqrt(K) * (2 ** bits_a / 3.46) * (2 ** bits_w / 3.46) * 3e-3))   # y of order 1
    y = orc.qlinear(qa, s_a, z_a, lin)
    a_off = b.store_offset(bits_a, z_a)
    A = dev((qa - a_off).astype(np.int8))
    rs = torch.empty(M, dtype=torch.int32, device="cuda")
    b.rq_rowsum_i8(ctx, A, rs)
    if act == "none3":
        seg = N // 3
        s_o, z_o, want = [], [], np.empty((M, N), np.int64)
        for i in range(3):
            part = y[:, i * seg:(i + 1) * seg]
            s = np.float32((part.max() - part.min()) / (2 ** bits_o - 1))
            z = int(np.rint(-part.min() / np.float64(s)))
            s_o.append(float(s)); z_o.append(z)
            want[:, i * seg:(i + 1) * seg] = orc.uniform_quant(part, s, z, bits_o)
        off_o = [b.store_offset(bits_o, z) for z in z_o]
        out = torch.zeros((M, N), dtype=torch.int8, device="cuda")
        b.rq_qgemm(ctx, A, a_off, z_a, float(s_a), lin_to_device(lin, bits_w), out_q=out, bits_o=bits_o, s_o=s_o, z_o=z_o,
                   off_o=off_o, seg_len=seg, rowsum_a=rs)
        got = out.cpu().numpy().astype(np.int64)
        for i in range(3):
            got[:, i * seg:(i + 1) * seg] += off_o[i]
    else:
        Dm = N // 2
        hid = orc.mlp_activation(y, orc.ACT_GELU if act == "gelu" else orc.ACT_SILU_GATED, Dm)
        s = np.float32((hid.max() - hid.min()) / (2 ** bits_o - 1))
        z = int(np.rint(-hid.min() / np.float64(s)))
        want = orc.uniform_quant(hid, s, z, bits_o)
        off = b.store_offset(bits_o, z)
        out = torch.zeros(want.shape, dtype=torch.int8, device="cuda")
        outf = None if q_only else torch.zeros(want.shape, dtype=torch.float32, device="cuda")
        b.rq_qgemm(ctx, A, a_off, z_a, float(s_a), lin_to_device(lin, bits_w, Dm if act == "gated" else 0),
                   act=b.ACT_GELU if act == "gelu" else b.ACT_SILU_GATED, out_q=out, out_f32=outf, bits_o=bits_o, s_o=[float(s)],
                   z_o=[z], off_o=[off], seg_len=want.shape[1], rowsum_a=rs)
        if not q_only:
            assert_float_close(outf.cpu().numpy(), hid, "activation " + act)
        got = out.cpu().numpy().astype(np.int64) + off
    assert_codes_close(got, want, "requant %s b%d" % (act, bits_o))


@pytest.mark.parametrize("M,N,K", [(1, 768, 768), (3, 2304, 768), (16, 1024, 4096), (2, 512, 11008), (1, 96, 64), (5, 4096, 2112)])
@pytest.mark.parametrize("bits_a", [8, 4])
def test_few_token_path_w4(rq, M, N, K, bits_a):
    """M <= 12 with packed 4-bit weights takes the matrix-vector kernel (16 takes the MFMA kernel): accumulators bit-exact, float output and
    re-quantized codes against the oracle's linear."""
    b, ctx = rq
    print("case", M, N, K, bits_a, flush=True)
    g = np.random.default_rng(M * 7 + N + K + bits_a)
    qa, z_a = _act_codes(g, M, K, bits_a)
    lin = random_linear(g, N, K, 4)
    want_acc = orc.qlinear_acc(qa, z_a, lin["codes"], lin["z_w"])
    s_a = np.float32(0.02)
    y = orc.qlinear(qa, s_a, z_a, lin)
    res = g.normal(size=(M, N)).astype(np.float32)
    a_off = b.store_offset(bits_a, z_a)
    A = dev((qa - a_off).astype(np.int8))
    rs = torch.empty(M, dtype=torch.int32, device="cuda")
    b.rq_rowsum_i8(ctx, A, rs)
    acc = torch.full((M, N), -7, dtype=torch.int32, device="cuda")
    outf = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    ld = lin_to_device(lin, 4)
    b.rq_qgemm(ctx, A, a_off, z_a, float(s_a), ld, out_acc=acc, out_f32=outf, residual=dev(res), rowsum_a=rs)
    torch.cuda.synchronize()
    assert np.array_equal(acc.cpu().numpy().astype(np.int64), want_acc)
    assert_float_close(outf.cpu().numpy(), y + res, "few-token f32")
    s_o = np.float32((y.max() - y.min()) / 255)
    z_o = int(np.rint(-y.min() / np.float64(s_o)))
    off_o = b.store_offset(8, z_o)
    outq = torch.zeros((M, N), dtype=torch.int8, device="cuda")
    b.rq_qgemm(ctx, A, a_off, z_a, float(s_a), ld, out_q=outq, bits_o=8, s_o=[float(s_o)], z_o=[z_o], off_o=[off_o], seg_len=N, rowsum_a=rs)
    # a handful of outputs: one float32-vs-float64 near-tie is allowed even when it exceeds 1e-4 of so few elements
    assert_codes_close(outq.cpu().numpy().astype(np.int64) + off_o, orc.uniform_quant(y, s_o, z_o, 8), "few-token codes",
                       budget=max(1e-4, 1.5 / (M * N)))


@pytest.mark.parametrize("act", ["gelu", "gated"])
def test_few_token_path_activations(rq, act):
    b, ctx = rq
    M, K = 4, 512
    N = 384 if act == "gelu" else 512
    g = np.random.default_rng(77 + len(act))
    qa, z_a = _act_codes(g, M, K, 8)
    lin = random_linear(g, N, K, 4)
    s_a = np.float32(1.5 / (np.sqrt(K) * (256 / 3.46) * (16 / 3.46) * 3e-3))
    y = orc.qlinear(qa, s_a, z_a, lin)
    Dm = N // 2
    hid = orc.mlp_activation(y, orc.ACT_GELU if act == "gelu" else orc.ACT_SILU_GATED, Dm)
    a_off = b.store_offset(8, z_a)
    A = dev((qa - a_off).astype(np.int8))
    rs = torch.empty(M, dtype=torch.int32, device="cuda")
    b.rq_rowsum_i8(ctx, A, rs)
    outf = torch.zeros(hid.shape, dtype=torch.float32, device="cuda")
    b.rq_qgemm(ctx, A, a_off, z_a, float(s_a), lin_to_device(lin, 4, Dm if act == "gated" else 0),
               act=b.ACT_GELU if act == "gelu" else b.ACT_SILU_GATED, out_f32=outf, rowsum_a=rs)
    assert_float_close(outf.cpu().numpy(), hid, "few-token " + act)


@pytest.mark.parametrize("M,N,K,bits,kind", [(197, 768, 768, 4, 0), (64, 256, 128, 4, 0), (333, 512, 3072, 6, 1), (1, 768, 64, 4, 0),
                                             (130, 768, 1536, 4, 1)])
def test_gemm_with_layernorm_quant_epilogue(rq, M, N, K, bits, kind):
    """rq_qgemm_ln_quant: xbar = linear + residual against the oracle's linear, and the codes against the oracle's
    LayerNorm / RMSNorm quantizer applied to the oracle's xbar."""
    from tests.helpers import folded_ln_case
    b, ctx = rq
    print("case", M, N, K, bits, kind, flush=True)
    g = np.random.default_rng(M + N + K)
    qa, z_a = _act_codes(g, M, K, 4)
    lin = random_linear(g, N, K, 4)
    s_a = np.float32(0.05)
    res = (g.normal(size=(M, N)) * np.exp(1.5 * g.normal(size=N))[None, :]).astype(np.float32)
    xbar = orc.qlinear(qa, s_a, z_a, lin) + res
    # a folded affine and layer-wise quantizer calibrated on these rows (plus spare rows so that a single row calibrates too)
    cal = np.concatenate([xbar, (g.normal(size=(40, N)) * np.abs(xbar).mean(axis=0)[None, :])], axis=0)
    c = folded_ln_case(cal.astype(np.float32), 3, bits, kind)
    want = orc.ln_quant(xbar, c["gamma_t"], c["beta_t"], c["s_t"], c["z_t"], bits, 1e-6, kind)
    a_off = b.store_offset(4, z_a)
    A = dev((qa - a_off).astype(np.int8))
    outf = torch.zeros((M, N), dtype=torch.float32, device="cuda")
    q = torch.zeros((M, N), dtype=torch.int8, device="cuda")
    off = b.rq_qgemm_ln_quant(ctx, A, a_off, z_a, float(s_a), lin_to_device(lin, 4), dev(res), outf, dev(c["gamma_t"]),
                              None if c["beta_t"] is None else dev(c["beta_t"]), float(c["s_t"]), int(c["z_t"]), bits, q,
                              norm_kind=kind)
    assert_float_close(outf.cpu().numpy(), xbar, "xbar")
    got = q.cpu().numpy().astype(np.int64) + off
    assert_codes_close(got, want, "codes after the fused normalization", budget=max(1e-4, 1.5 / (M * N)))

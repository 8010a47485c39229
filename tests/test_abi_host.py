"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared entry point, the
Python structures have the C layout, and every call validates its arguments before touching a device."""
import ctypes as C
import os
import re
import subprocess
import sys

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "repquant.h")


@pytest.fixture(scope="module")
def b():
    from paper_2402_05628_amd import binding
    return binding


@pytest.fixture()
def host_ctx(b):
    ctx = b.Context(None)        # host-only context: validation runs, valid calls return RQ_ERR_UNSUPPORTED
    yield ctx
    ctx.close()


def _declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^(?:rq_status|size_t|int32_t|void|const char\*)\s+(rq_\w+)\s*\(", text, flags=re.M)
    assert len(names) >= 20
    return names


def test_every_declared_symbol_is_exported(b):
    missing = [n for n in _declared_functions() if not hasattr(b.lib, n)]
    assert not missing, missing


def test_named_hot_path_calls_are_declared():
    names = set(_declared_functions())
    for n in ("rq_reparam_fold", "rq_ln_quant", "rq_qgemm", "rq_softmax_log2_quant", "rq_attn_pv", "rq_block_forward"):
        assert n in names


def test_structures_have_the_c_layout(b, tmp_path):
    """sizeof and the offset of the last field of every descriptor, as gcc lays the header out."""
    pairs = [("rq_fold_desc", b.FoldDesc), ("rq_wq_desc", b.WqDesc), ("rq_ln_desc", b.LnDesc), ("rq_gemm_desc", b.GemmDesc),
             ("rq_softmax_desc", b.SoftmaxDesc), ("rq_qk_softmax_desc", b.QkSoftmaxDesc), ("rq_attn_fused_desc", b.AttnFusedDesc),
             ("rq_pv_desc", b.PvDesc), ("rq_dual_clip_desc", b.DualClipDesc), ("rq_gptq_desc", b.GptqDesc),
             ("rq_qlinear", b.QLinear), ("rq_block_params", b.BlockParams), ("rq_block_raw", b.BlockRaw),
             ("rq_block_layout", b.BlockLayout), ("rq_blob_header", b.BlobHeader)]
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "repquant.h"', "int main(void) {"]
    for cname, cls in pairs:
        last = cls._fields_[-1][0]
        lines.append('  printf("%s %%zu %%zu\\n", sizeof(%s), offsetof(%s, %s));' % (cname, cname, cname, last))
    lines += ["  return 0;", "}"]
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    got = {l.split()[0]: (int(l.split()[1]), int(l.split()[2])) for l in out if l.strip()}
    for cname, cls in pairs:
        last = cls._fields_[-1][0]
        assert got[cname] == (C.sizeof(cls), getattr(cls, last).offset), cname


def test_header_compiles_as_plain_c(tmp_path):
    src = tmp_path / "plain.c"
    src.write_text('#include "repquant.h"\nint main(void) { return (int)RQ_OK; }\n')
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"), str(src), "-o",
                    str(tmp_path / "plain")], check=True)


def test_store_offset_rule(b):
    # off = z when code - z fits int8 for every code, otherwise 128
    for bits in range(2, 9):
        for z in range(0, 2 ** bits):
            off = b.store_offset(bits, z)
            lo, hi = -off, 2 ** bits - 1 - off
            assert -128 <= lo and hi <= 127
            if -z >= -128 and 2 ** bits - 1 - z <= 127:
                assert off == z
            else:
                assert off == 128


FAKE = 0x10000     # non-NULL, 64 KiB aligned: never dereferenced, validation fails or the host-only context refuses first


def _ln_desc(b, **kw):
    d = b.LnDesc(T=4, D=64, norm_kind=b.NORM_LAYERNORM, eps=1e-6, x=FAKE, ldx=64, gamma_t=FAKE, beta_t=FAKE, s_tilde=0.1,
                 z_tilde=3, bits=4, store_off=3, q=FAKE, ldq=64, rowsum=None)
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def _status(b, ctx, fn, desc):
    return fn(ctx.handle, C.byref(desc))


def test_ln_quant_validation(b, host_ctx):
    fn = b.lib.rq_ln_quant
    assert _status(b, host_ctx, fn, _ln_desc(b)) == 3                   # valid: refused only for lack of a device
    assert "host-only" in b.lib.rq_last_error(host_ctx.handle).decode() or b.lib.rq_last_error(host_ctx.handle)
    assert _status(b, host_ctx, fn, _ln_desc(b, x=None)) == 1
    assert _status(b, host_ctx, fn, _ln_desc(b, bits=9)) == 1
    assert _status(b, host_ctx, fn, _ln_desc(b, bits=1)) == 1
    assert _status(b, host_ctx, fn, _ln_desc(b, s_tilde=0.0)) == 1
    assert _status(b, host_ctx, fn, _ln_desc(b, s_tilde=float("nan"))) == 1
    assert _status(b, host_ctx, fn, _ln_desc(b, D=66)) == 2             # D % 4
    assert _status(b, host_ctx, fn, _ln_desc(b, ldx=32)) == 2           # pitch below D
    assert _status(b, host_ctx, fn, _ln_desc(b, T=-1)) == 2
    assert _status(b, host_ctx, fn, _ln_desc(b, x=FAKE + 4)) == 1       # misaligned
    assert _status(b, host_ctx, fn, _ln_desc(b, store_off=200)) == 1    # code - off would not fit int8
    msg = b.lib.rq_last_error(host_ctx.handle).decode()
    assert "rq_ln_quant" in msg


def test_null_context_and_null_descriptor(b, host_ctx):
    assert b.lib.rq_ln_quant(None, C.byref(_ln_desc(b))) == 1
    assert b.lib.rq_ln_quant(host_ctx.handle, None) == 1
    assert b.lib.rq_qgemm(host_ctx.handle, None) == 1
    assert b.lib.rq_softmax_log2_quant(host_ctx.handle, None) == 1
    assert b.lib.rq_attn_pv(host_ctx.handle, None) == 1
    assert b.lib.rq_reparam_fold(host_ctx.handle, None) == 1
    assert len(b.lib.rq_last_error(None)) > 0


def _gemm_desc(b, **kw):
    d = b.GemmDesc()
    d.M, d.N, d.K = 64, 64, 64
    d.A, d.lda, d.a_off, d.z_a, d.s_a = FAKE, 64, 8, 8, 0.1
    d.B, d.ldb, d.b_format = FAKE, 64, b.W_I8_BAKED
    d.s_b, d.z_b, d.colsum_b = FAKE, FAKE, FAKE
    d.batch_outer, d.batch_inner, d.n_seg = 1, 1, 1
    d.out_f32, d.ldf = FAKE, 64
    for k, v in kw.items():
        setattr(d, k, v)
    return d


def test_qgemm_validation(b, host_ctx):
    fn = b.lib.rq_qgemm
    assert _status(b, host_ctx, fn, _gemm_desc(b)) == 3
    assert _status(b, host_ctx, fn, _gemm_desc(b, A=None)) == 1
    assert _status(b, host_ctx, fn, _gemm_desc(b, out_f32=None)) == 1        # no output requested
    assert _status(b, host_ctx, fn, _gemm_desc(b, K=60)) == 2                # K % 64
    assert _status(b, host_ctx, fn, _gemm_desc(b, lda=32)) == 2
    assert _status(b, host_ctx, fn, _gemm_desc(b, b_format=7)) == 1
    assert _status(b, host_ctx, fn, _gemm_desc(b, s_a=-1.0)) == 1
    assert _status(b, host_ctx, fn, _gemm_desc(b, b_format=b.W_U4, ldb=16)) == 2    # packed rows hold K/2 bytes
    assert _status(b, host_ctx, fn, _gemm_desc(b, b_format=b.W_I8_CENTERED)) == 1   # centered weights need rowsum_a
    assert _status(b, host_ctx, fn, _gemm_desc(b, act=5)) == 1


def test_qgemm_ln_quant_validation(b, host_ctx):
    fn = b.lib.rq_qgemm_ln_quant
    def call(g=None, l=None):
        gd = _gemm_desc(b, **{**dict(M=4, N=256, K=64, b_format=b.W_U4, ldb=32, residual=FAKE, ldr=256, ldf=256), **(g or {})})
        ld = _ln_desc(b, **{**dict(T=4, D=256, x=None, ldx=256, ldq=256), **(l or {})})
        return fn(host_ctx.handle, C.byref(gd), C.byref(ld))
    assert call() == 3                                           # valid, refused only for lack of a device
    assert "host-only" in b.lib.rq_last_error(host_ctx.handle).decode()
    assert fn(host_ctx.handle, C.byref(_gemm_desc(b)), None) == 1
    assert call(l={"T": 5}) == 2                                 # the two descriptors disagree on the shape
    assert call(l={"bits": 9}) == 1
    assert call(g={"residual": None}) == 3                       # the fused kernel covers only the residual form
    assert "rq_qgemm + rq_ln_quant" in b.lib.rq_last_error(host_ctx.handle).decode()
    assert call(g={"b_format": b.W_I8_BAKED, "ldb": 64}) == 3
    assert call(l={"bits": 8, "store_off": 128}) == 3
    assert call(g={"K": 60}) == 2


def test_dual_clip_validation(b, host_ctx):
    fn = b.lib.rq_dual_clip_learn
    def call(**kw):
        f = dict(T=100, D=64, ldx=64, x=FAKE, norm_kind=b.NORM_LAYERNORM, eps=1e-6, gamma=FAKE, beta=None, bits=4, iters=100,
                 lr=0.01, alpha0=4.0, alpha1=FAKE, alpha2=FAKE, workspace=FAKE, workspace_bytes=b.lib.rq_dual_clip_workspace_bytes(100))
        f.update(kw)
        return fn(host_ctx.handle, C.byref(b.DualClipDesc(**f)))
    assert b.lib.rq_dual_clip_workspace_bytes(100) == 1600
    assert call() == 3                                              # valid: refused only for lack of a device
    assert call(gamma=None, workspace=None, workspace_bytes=0, D=7, ldx=7) == 3     # x given as X': no workspace, any D
    assert fn(host_ctx.handle, None) == 1
    assert call(x=None) == 1 and call(alpha1=None) == 1
    assert call(bits=1) == 1 and call(bits=17) == 1
    assert call(iters=-1) == 1 and call(lr=0.0) == 1 and call(lr=float("nan")) == 1
    assert call(T=0) == 2 and call(ldx=32) == 2 and call(D=66, ldx=68) == 2
    assert call(workspace_bytes=8) == 4 and call(workspace=None) == 4
    assert "rq_dual_clip_learn" in b.lib.rq_last_error(host_ctx.handle).decode()
    assert call(alpha1=FAKE + 4) == 1


def test_gptq_validation(b, host_ctx):
    fn = b.lib.rq_gptq_quant_pack
    need = b.lib.rq_gptq_workspace_bytes(128, 64, 300)
    assert need > 128 * 64 * 8 + 3 * 64 * 64 * 8
    big = FAKE & ~0xFF
    def call(**kw):
        f = dict(N=128, K=64, bits=4, format=b.W_U4, gate_up_rows=0, W=FAKE, bias=None, A=FAKE, T=300, lda=64, a_off=8, z_a=8,
                 percdamp=0.01, w_out=FAKE, s_w=FAKE, z_w=FAKE, colsum_w=FAKE, bias_out=None, workspace=big, workspace_bytes=need)
        f.update(kw)
        return fn(host_ctx.handle, C.byref(b.GptqDesc(**f)))
    assert call() == 3
    assert fn(host_ctx.handle, None) == 1
    assert call(A=None) == 1 and call(W=None) == 1
    assert call(K=96, lda=96) == 2 and call(K=16384, lda=16384) == 2       # K % 64, K <= 8192
    assert call(T=0) == 2 and call(T=200000) == 2 and call(lda=32) == 2
    assert call(bits=5) == 1                                               # packed 4-bit format needs bits = 4
    assert call(format=b.W_I8_BAKED, bits=8) == 1 and call(format=9) == 1
    assert call(gate_up_rows=48) == 2
    assert call(percdamp=0.0) == 1
    assert call(workspace_bytes=need - 1) == 4 and call(workspace=big + 8) == 4
    assert "rq_gptq_quant_pack" in b.lib.rq_last_error(host_ctx.handle).decode()


def test_percentile_validation(b, host_ctx):
    fn = b.lib.rq_ln_channel_percentile
    def call(x=FAKE, T=100, D=64, ldx=64, kind=0, eps=1e-6, gamma=FAKE, q=(0.01, 0.99), lo=FAKE, hi=FAKE, ws=FAKE, nbytes=1600):
        return fn(host_ctx.handle, x, T, D, ldx, kind, eps, gamma, None, q[0], q[1], lo, hi, ws, nbytes)
    assert call() == 3
    assert call(gamma=None, ws=None, nbytes=0, D=7, ldx=7) == 3
    assert call(x=None) == 1 and call(lo=None) == 1
    assert call(q=(0.6, 0.4)) == 1 and call(q=(-0.1, 0.5)) == 1 and call(q=(0.5, 1.5)) == 1
    assert call(T=0) == 2 and call(ldx=32) == 2 and call(D=66, ldx=68) == 2
    assert call(nbytes=100) == 4 and call(kind=3) == 1 and call(eps=0.0) == 1


def test_softmax_and_pv_validation(b, host_ctx):
    sd = dict(G=2, H=2, Nq=8, Nk=8, ld=16, acc=FAKE, logit_scale=0.1, bias=None, mask=0, s_log=1.0, bits=4, codes=FAKE)
    ok = b.SoftmaxDesc(**sd)
    assert b.lib.rq_softmax_log2_quant(host_ctx.handle, C.byref(ok)) == 3
    for k, v, want in (("bits", 9, 1), ("ld", 6, 2), ("ld", 8200, 2), ("s_log", 0.0, 1), ("logit_scale", -1.0, 1), ("mask", 3, 1),
                       ("acc", None, 1), ("Nk", 0, 2)):
        bad = b.SoftmaxDesc(**{**sd, k: v})
        assert b.lib.rq_softmax_log2_quant(host_ctx.handle, C.byref(bad)) == want, (k, v)
    causal = b.SoftmaxDesc(**{**sd, "mask": 1, "Nq": 4})
    assert b.lib.rq_softmax_log2_quant(host_ctx.handle, C.byref(causal)) == 2

    pd = dict(batch=1, H=2, Nq=8, Nk=8, d_head=32, ld=16, codes=FAKE, V=FAKE, ldv=192, s_log=1.0, s_v=0.1, z_v=3, v_off=3, bits_p=4,
              mask=0, out_f32=FAKE, ldf=64)
    assert b.lib.rq_attn_pv(host_ctx.handle, C.byref(b.PvDesc(**pd))) == 3
    for k, v, want in (("d_head", 48, 2), ("ld", 8, 2), ("bits_p", 1, 1), ("s_v", 0.0, 1), ("V", None, 1), ("out_f32", None, 1),
                       ("ldv", 32, 2)):
        bad = b.PvDesc(**{**pd, k: v})
        assert b.lib.rq_attn_pv(host_ctx.handle, C.byref(bad)) == want, (k, v)

    qd = dict(batch=1, H=2, N=8, d_head=32, Q=FAKE, K=FAKE, ld_tok=192, q_off=3, z_q=3, k_off=3, z_k=3, logit_scale=0.1, bias=None,
              mask=0, s_log=1.0, bits=4, codes=FAKE, ld=16)
    assert b.lib.rq_qk_softmax_log2_quant(host_ctx.handle, C.byref(b.QkSoftmaxDesc(**qd))) == 3
    for k, v, want in (("N", 70000, 2), ("d_head", 48, 2), ("ld", 8, 2), ("bits", 0, 1), ("Q", None, 1), ("ld_tok", 40, 2)):
        bad = b.QkSoftmaxDesc(**{**qd, k: v})
        assert b.lib.rq_qk_softmax_log2_quant(host_ctx.handle, C.byref(bad)) == want, (k, v)
    # rows beyond 288 keys: accepted without a bias, refused with one
    long_row = {**qd, "N": 300, "ld": 304}
    assert b.lib.rq_qk_softmax_log2_quant(host_ctx.handle, C.byref(b.QkSoftmaxDesc(**long_row))) == 3
    assert b.lib.rq_qk_softmax_log2_quant(host_ctx.handle, C.byref(b.QkSoftmaxDesc(**{**long_row, "bias": FAKE}))) == 2


def test_attn_fused_validation(b, host_ctx):
    fd = dict(batch=1, H=2, N=64, d_head=64, Q=FAKE, K=FAKE, V=FAKE, ld_tok=384, q_off=3, z_q=3, k_off=3, z_k=3, v_off=3, z_v=3,
              logit_scale=0.1, s_log=1.0, s_v=0.1, bits_p=4, codes=None, ld=0, out_f32=FAKE, ldf=128)
    assert b.lib.rq_attn_fused(host_ctx.handle, C.byref(b.AttnFusedDesc(**fd))) == 3
    for k, v, want in (("N", 320, 2), ("bits_p", 7, 2), ("d_head", 48, 2), ("V", None, 1), ("out_f32", None, 1), ("s_v", 0.0, 1),
                       ("ld_tok", 100, 2), ("ldf", 64, 2)):
        assert b.lib.rq_attn_fused(host_ctx.handle, C.byref(b.AttnFusedDesc(**{**fd, k: v}))) == want, (k, v)
    assert b.attn_fused_supported(197, 64, 4) and b.attn_fused_supported(257, 64, 4) and not b.attn_fused_supported(197, 64, 6)
    # with a bias and / or codes of 5 or 6 bits: rows of up to 160 keys
    assert b.attn_fused_supported(49, 32, 6, True) and b.attn_fused_supported(160, 64, 5) and not b.attn_fused_supported(161, 64, 4, True)
    assert not b.attn_fused_supported(49, 32, 7) and not b.attn_fused_supported(49, 32, 8, True)
    assert b.attn_fused_supported(288, 128, 4) and not b.attn_fused_supported(289, 32, 4) and b.attn_fused_supported(96, 128, 4)


def test_fold_and_weight_pack_validation(b, host_ctx):
    fd = dict(D=64, D_out=32, s_ch=FAKE, z_ch=FAKE, gamma=FAKE, beta=FAKE, W=FAKE, b=FAKE, s_log=1.0, s_tilde=FAKE, z_tilde=FAKE,
              gamma_t=FAKE, beta_t=FAKE, W_t=FAKE, b_t=FAKE, s_log_pair=None)
    assert b.lib.rq_reparam_fold(host_ctx.handle, C.byref(b.FoldDesc(**fd))) == 3
    for k, v, want in (("D", 0, 2), ("s_ch", None, 1), ("gamma_t", None, 1)):
        assert b.lib.rq_reparam_fold(host_ctx.handle, C.byref(b.FoldDesc(**{**fd, k: v}))) == want, (k, v)
    wq = b.WqDesc()
    assert b.lib.rq_weight_quant_pack(host_ctx.handle, C.byref(wq)) in (1, 2)      # all-zero descriptor


def test_block_forward_validation(b, host_ctx):
    p = b.BlockParams()
    assert b.lib.rq_block_workspace_bytes(C.byref(p), 1, 8) == 0          # D = 0
    rc = b.lib.rq_block_forward(host_ctx.handle, C.byref(p), C.c_void_p(FAKE), C.c_void_p(FAKE), 1, 8, C.c_void_p(FAKE), 1 << 20)
    assert rc in (1, 2)
    assert "rq_block_forward" in b.lib.rq_last_error(host_ctx.handle).decode()
    assert b.lib.rq_block_forward(None, C.byref(p), None, None, 1, 8, None, 0) == 1
    h = host_ctx.handle
    assert b.lib.rq_set_gemm_tile(h, 99) == 1 and b.lib.rq_set_gemm_tile(h, 9) == 1 and b.lib.rq_set_gemm_tile(None, 0) == 1
    assert b.lib.rq_set_gemm_tile(h, 8) == 0 and b.lib.rq_set_gemm_tile(h, 256 + 5) == 0 and b.lib.rq_set_gemm_tile(h, 512 + 3) == 0 and b.lib.rq_set_gemm_tile(h, 800) == 1
    assert b.lib.rq_set_gemm_tile(h, 0) == 0      # 8: the 256 x 256 tiles; + 256: no raw-nibble variant
    assert b.lib.rq_set_block_streams(h, 0) == 1 and b.lib.rq_set_block_streams(h, 4) == 1 and b.lib.rq_set_block_streams(None, 1) == 1
    assert b.lib.rq_set_block_streams(h, 1) == 0 and b.lib.rq_set_block_streams(h, 3) == 0 and b.lib.rq_set_block_streams(h, 2) == 0


def test_workspace_bytes_grow_with_the_problem(b):
    def params(D, H, Dm):
        p = b.BlockParams()
        p.D, p.H, p.Dm = D, H, Dm
        return p
    small = b.lib.rq_block_workspace_bytes(C.byref(params(384, 6, 1536)), 1, 197)
    big = b.lib.rq_block_workspace_bytes(C.byref(params(768, 12, 3072)), 64, 197)
    assert 0 < small < big
    # ViT-B at batch 64: int8 activations, the float residual stream and the attention scratch stay far below HBM size
    assert big < (1 << 30)


def test_calibration_plan_keeps_logits_and_codes_apart(b):
    """The calibration always runs the three separate attention kernels: its plan must hold int32 logits AND codes for one
    chunk, in regions of their own and inside the workspace it asks for, whatever the forward pass would choose for the
    shape (short unmasked rows take the one-kernel attention there and need neither).  Includes small-head long-row shapes
    and a chunk budget that splits the batch."""
    cases = [(768, 12, 3072, 64, 197, 0), (1024, 16, 4096, 128, 257, 0), (1024, 16, 4096, 128, 257, 1 << 20), (512, 4, 1024, 1, 2048, 0),
             (512, 4, 1024, 1, 4096, 0), (128, 4, 512, 64, 49, 1 << 20), (384, 6, 1536, 1, 197, 0)]
    for D, H, Dm, batch, seq, chunk in cases:
        raw = b.BlockRaw()
        raw.D, raw.H, raw.Dm, raw.attn_chunk_bytes = D, H, Dm, chunk
        lay = b.BlockLayout()
        assert b.lib.rq_block_calibrate_workspace_layout(C.byref(raw), batch, seq, C.byref(lay)) == 0
        ld = (seq + 15) // 16 * 16
        assert lay.ld == ld and 1 <= lay.batch_chunk <= batch
        need_logits, need_codes = 4 * lay.batch_chunk * H * seq * ld, lay.batch_chunk * H * seq * ld
        assert lay.logits_bytes >= need_logits and lay.codes_bytes >= need_codes, (D, H, batch, seq)
        assert lay.codes - lay.logits >= need_logits                      # the codes start after the last logit
        assert lay.o - lay.codes >= need_codes                            # and end before the attention output
        regions = sorted([(lay.a, batch * seq * D), (lay.rowsum, 4 * batch * seq), (lay.qkv, 3 * batch * seq * D),
                          (lay.logits, need_logits), (lay.codes, need_codes), (lay.o, batch * seq * D),
                          (lay.xbar, 4 * batch * seq * D), (lay.hidden, batch * seq * Dm)])
        for (o0, n0), (o1, _) in zip(regions, regions[1:]):
            assert o0 + n0 <= o1, (D, H, batch, seq)
        total = b.lib.rq_block_calibrate_workspace_bytes(C.byref(raw), batch, seq)
        assert total == lay.total and regions[-1][0] + regions[-1][1] <= total
        if chunk:
            assert lay.batch_chunk < batch                                # the budget splits this batch
    # the forward plan of a short unmasked row keeps neither logits nor codes in memory
    p = b.BlockParams()
    p.D, p.H, p.Dm, p.bits_p = 768, 12, 3072, 4
    lay = b.BlockLayout()
    assert b.lib.rq_block_workspace_layout(C.byref(p), 64, 197, C.byref(lay)) == 0
    assert lay.logits_bytes == 0 and lay.codes_bytes == 0 and lay.batch_chunk == 64
    p.attn_path = b.ATTN_THREE_KERNELS
    assert b.lib.rq_block_workspace_layout(C.byref(p), 64, 197, C.byref(lay)) == 0
    assert lay.logits_bytes >= 4 * lay.batch_chunk * 12 * 197 * 208 and lay.codes - lay.logits >= lay.logits_bytes
    assert b.lib.rq_block_workspace_layout(None, 64, 197, C.byref(lay)) == 1


def test_synthetic_inputs_are_seeded_and_shaped():
    from paper_2402_05628_amd import synth
    cfg = synth.CONFIGS[0]
    a, c = synth.make_block(cfg, 0, 0), synth.make_block(cfg, 0, 0)
    d = synth.make_block(cfg, 0, 1)
    for k, v in a.items():
        if v is None:
            assert c[k] is None
            continue
        assert np.array_equal(v, c[k]), k
    assert not np.array_equal(a["x"], d["x"])
    assert a["x"].shape == (cfg.tokens, cfg.D) and a["x"].dtype == np.float32
    assert a["w_qkv"].shape == (3 * cfg.D, cfg.D) and a["w_fc2"].shape == (cfg.D, cfg.Dm)
    # the LN input carries a few channels tens of times larger than the median channel
    ch = np.abs(a["x"]).mean(axis=0)
    assert ch.max() / np.median(ch) > 20
    shapes = [(c_.batch, c_.seq, c_.D, c_.H, c_.Dm) for c_ in synth.CONFIGS]
    assert shapes[1] == (64, 197, 768, 12, 3072)
    assert shapes[3][1:] == (2048, 4096, 32, 11008)


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2402_05628_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert not re.search(r"^\s*(from|import)\s+oracle|#include\s+\"[^\"]*oracle", text, flags=re.M), os.path.join(dirpath, f)
    for f in ("paper_2402_05628_amd/binding.py", "paper_2402_05628_amd/__init__.py", "paper_2402_05628_amd/_build.py"):
        assert "oracle" not in open(os.path.join(ROOT, f)).read().lower(), f


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr or "one GPU" in r.stderr


def _fake_block_params(b, rel_bias=False, rms=False):
    bp = b.BlockParams()
    bp.D, bp.H, bp.Dm, bp.bits_a, bp.bits_p, bp.eps = 64, 2, 128, 4, 4, 1e-6
    for k in ("ln1_gamma_t", "ln2_gamma_t"):
        setattr(bp, k, FAKE)
    if not rms:
        bp.ln1_beta_t, bp.ln2_beta_t = FAKE, FAKE

    def lin(N, K, fmt):
        q = b.QLinear()
        q.N, q.K, q.bits, q.format = N, K, 4, fmt
        q.w, q.s_w, q.z_w, q.colsum_w, q.bias = FAKE, FAKE, FAKE, FAKE, FAKE
        return q
    bp.qkv, bp.proj, bp.fc1, bp.fc2 = lin(192, 64, b.W_U4), lin(64, 64, b.W_I8_BAKED), lin(128, 64, b.W_U4), lin(64, 128, b.W_I8_CENTERED)
    if rel_bias:
        bp.rel_bias = FAKE
    return bp


def _up(n):
    return (n + 255) // 256 * 256


def test_block_blob_size_is_the_header_plus_the_aligned_arrays(b):
    bp = _fake_block_params(b)
    want = _up(C.sizeof(b.BlobHeader)) + 4 * _up(64 * 4)
    for N, K, packed in ((192, 64, True), (64, 64, False), (128, 64, True), (64, 128, False)):
        want += _up(N * K // 2 if packed else N * K) + 4 * _up(N * 4)
    assert b._rq_blob_bytes(C.byref(bp), 0) == want
    # a relative-position bias adds its elements; it needs a positive count
    bpr = _fake_block_params(b, rel_bias=True)
    assert b._rq_blob_bytes(C.byref(bpr), 2 * 49 * 49) == want + _up(2 * 49 * 49 * 4)
    assert b._rq_blob_bytes(C.byref(bpr), 0) == 0
    # RMSNorm blocks have no beta~: two arrays fewer
    assert b._rq_blob_bytes(C.byref(_fake_block_params(b, rms=True)), 0) == want - 2 * _up(64 * 4)
    # a required array missing, or no parameters at all: no blob
    bad = _fake_block_params(b)
    bad.qkv.s_w = None
    assert b._rq_blob_bytes(C.byref(bad), 0) == 0
    assert b._rq_blob_bytes(None, 0) == 0
    odd = _fake_block_params(b)
    odd.qkv.K = 63
    assert b._rq_blob_bytes(C.byref(odd), 0) == 0      # packed 4-bit rows need an even K


def _blob_image(b, **edits):
    """A well-formed blob (zero arrays) of the fake block, built here field by field, then edited."""
    h = b.BlobHeader()
    h.magic, h.header_bytes, h.version = b"RQBLOCK", C.sizeof(b.BlobHeader), 1
    h.D, h.H, h.Dm, h.bits_a, h.bits_p, h.eps = 64, 2, 128, 4, 4, 1e-6
    shapes = ((192, 64, b.W_U4), (64, 64, b.W_I8_BAKED), (128, 64, b.W_U4), (64, 128, b.W_I8_CENTERED))
    o = _up(C.sizeof(b.BlobHeader))
    lens = [64 * 4] * 4
    for k, (N, K, fmt) in enumerate(shapes):
        h.lin[k][0], h.lin[k][1], h.lin[k][2], h.lin[k][3] = N, K, 4, fmt
        lens += [N * K // 2 if fmt == b.W_U4 else N * K] + [N * 4] * 4
    lens.append(0)
    for i, n in enumerate(lens):
        h.off[i], h.len[i] = (o, n) if n else (0, 0)
        o += _up(n)
    h.total_bytes = o
    for k, v in edits.items():
        if k.startswith("off") or k.startswith("len"):
            getattr(h, k[:3])[int(k[3:])] = v
        elif k.startswith("lin"):
            h.lin[int(k[3])][int(k[4])] = v
        else:
            setattr(h, k, v)
    return bytes(h) + bytes(o - C.sizeof(b.BlobHeader))


def test_block_blob_check_accepts_a_well_formed_blob_and_names_what_is_wrong_with_others(b):
    good = _blob_image(b)
    assert b.check_block_blob(good) == len(good)
    assert b.check_block_blob(good + b"tail") == len(good)          # a longer buffer is fine
    cases = [(dict(magic=b"RQBLOCX"), 1, "magic"), (dict(version=2), 3, "version"), (dict(header_bytes=600), 2, "header"),
             (dict(D=0), 2, "out of range"), (dict(lin00=-5), 2, "out of range"), (dict(lin03=9), 2, "format"),
             (dict(lin01=63), 2, "even K"), (dict(len5=100), 2, "array 5"), (dict(off6=8), 2, "array 6"),
             (dict(off7=1 << 40), 2, "array 7"), (dict(off4=0, len4=0), 2, "required array 4"),
             (dict(rel_bias_elems=-1), 2, "rel_bias_elems")]
    for edits, status, word in cases:
        with pytest.raises(b.RqError) as e:
            b.check_block_blob(_blob_image(b, **edits))
        assert e.value.status == status and word in str(e.value), (edits, str(e.value))
    # two arrays swapped in place: in range and aligned, but out of order (they would be allowed to overlap otherwise)
    h = b.BlobHeader.from_buffer_copy(good)
    with pytest.raises(b.RqError):
        b.check_block_blob(_blob_image(b, off5=h.off[6], off6=h.off[5]))
    with pytest.raises(b.RqError) as e:
        b.check_block_blob(good[:len(good) - 1])
    assert "truncated" in str(e.value)
    with pytest.raises(b.RqError):
        b.check_block_blob(good[:100])


def test_block_blob_save_and_load_validate_before_any_copy(b, host_ctx):
    bp = _fake_block_params(b)
    n = b._rq_blob_bytes(C.byref(bp), 0)
    buf = (C.c_char * n)()
    assert b._rq_blob_save(host_ctx.handle, C.byref(bp), 0, C.cast(buf, C.c_void_p), n - 1) == 4       # blob too small
    assert b._rq_blob_save(host_ctx.handle, C.byref(bp), 0, None, n) == 1
    assert b._rq_blob_save(None, C.byref(bp), 0, C.cast(buf, C.c_void_p), n) == 1
    assert b._rq_blob_save(host_ctx.handle, C.byref(bp), 0, C.cast(buf, C.c_void_p), n) == 3           # valid: host-only context
    good = _blob_image(b)
    img = C.create_string_buffer(good, len(good))
    out = b.BlockParams()
    assert b._rq_blob_load(host_ctx.handle, C.cast(img, C.c_void_p), len(good), FAKE, len(good), C.byref(out)) == 3
    assert b._rq_blob_load(host_ctx.handle, C.cast(img, C.c_void_p), len(good), FAKE + 4, len(good), C.byref(out)) == 1   # misaligned arena
    assert b._rq_blob_load(host_ctx.handle, C.cast(img, C.c_void_p), len(good), FAKE, len(good) - 1, C.byref(out)) == 4   # arena too small
    assert b._rq_blob_load(host_ctx.handle, C.cast(img, C.c_void_p), len(good), FAKE, len(good), None) == 1
    assert b._rq_blob_load(host_ctx.handle, C.cast(img, C.c_void_p), 50, FAKE, len(good), C.byref(out)) == 2

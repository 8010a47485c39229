"""Full-size workloads in the launch configuration bench.py times, checked on sampled sequences.

Batch items (images, windows) never interact, so the oracle evaluates a few whole sequences of the batch one by one with
the same calibrated parameters and the rows of those sequences are compared element by element."""
import dataclasses

import numpy as np
import pytest
import torch

from oracle import repquant_oracle as orc
from paper_2402_05628_amd import synth
from tests.helpers import block_to_device, cfg_dict, dev

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def rq():
    from paper_2402_05628_amd import binding
    return binding, binding.Context(0)


@pytest.mark.timeout(600)
@pytest.mark.parametrize("cfg_id,cal_batch", [(1, 4), (2, 64), (4, 2)])
def test_full_batch_sampled_sequences(rq, cfg_id, cal_batch):
    b, ctx = rq
    cfg = synth.CONFIGS[cfg_id]
    print("case", cfg.name, flush=True)
    cal_cfg = cfg.with_batch(cal_batch)
    raw_c = synth.make_block(cal_cfg, cfg_id, seed=1)
    P = orc.calibrate_block(raw_c, cfg_dict(cal_cfg))           # the oracle's parameters, handed to both sides
    g = synth.rng_for(cfg_id, seed=2)
    x = g.standard_normal((cfg.tokens, cfg.D), dtype=np.float32)
    # same input distribution as the calibration batch: reuse its per-channel scales through the calibration rows' statistics
    ch = np.abs(raw_c["x"]).mean(axis=0) / np.sqrt(2.0 / np.pi)
    x *= ch.astype(np.float32)[None, :]
    blk = b.Block(ctx, cfg, block_to_device(P))
    xd = dev(x)
    y = torch.zeros_like(xd)
    blk.forward(xd, y, cfg.batch, cfg.seq)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    assert np.isfinite(got).all()
    picks = sorted({0, cfg.batch // 3, cfg.batch // 2, cfg.batch - 1})
    rows = np.concatenate([np.arange(i * cfg.seq, (i + 1) * cfg.seq) for i in picks])
    Ps = dict(P)
    Ps["cfg"] = cfg_dict(cfg.with_batch(len(picks)))
    want = orc.block_forward(Ps, x[rows])
    ref = np.abs(want).max()
    err = np.abs(got[rows] - want).max()
    print("  %d sampled sequences of %d: max|d| / max|ref| = %.3g" % (len(picks), cfg.batch, err / ref), flush=True)
    assert err <= 1e-3 * ref
    bar = 1e-3 * np.maximum(np.abs(want), 1e-3 * ref)
    assert float(np.mean(np.abs(got[rows] - want) > bar)) < 0.02


@pytest.mark.timeout(900)
def test_llama_shape_full_size_stage_by_stage(rq):
    """The LLaMA-7B-shaped block (one 2048-token sequence, hidden 4096, causal, gated MLP, W4/A8) at full size.

    With ~1 % of the channels scaled 50-200x the attention logits span hundreds of units, so Softmax is close to an argmax
    and ONE rounding-tie flip in a Q or K code can move a row's winning key.  The 8-bit re-quantization of Q, K, V is
    therefore guarded against ties (float64 re-decision), and this test holds the block to the stated bar: every stage
    teacher-forced on the oracle's own intermediates (integer accumulators bit-exact, codes within the tie budget, floats to
    1e-3); every code tensor of the whole pass read back from the workspace and compared; the oracle's stages fed with the
    GPU's own codes must reproduce the GPU's floats to 1e-3; and end to end max|d| <= 1e-3 max|ref| on every row that holds
    no differing code at any stage (all rows when none differs; the differing codes are within the tie budget)."""
    import math
    from tests.helpers import assert_codes_close, assert_float_close, lin_to_device
    b, ctx = rq
    cfg_id = 3
    cfg = synth.CONFIGS[cfg_id]
    raw_c = synth.make_block(cfg, cfg_id, seed=1)
    P = orc.calibrate_block(raw_c, cfg_dict(cfg))
    x = synth.rng_for(cfg_id, seed=2).standard_normal((cfg.tokens, cfg.D), dtype=np.float32)
    y_ref, t = orc.block_forward(P, x, keep=True)
    T, D, H, N, Dm = cfg.tokens, cfg.D, cfg.H, cfg.seq, cfg.Dm
    dh, ba, bp, bw = D // H, cfg.bits_a, cfg.bits_p, cfg.bits_w
    ln1, ln2 = P["ln1"], P["ln2"]
    q = torch.empty((T, D), dtype=torch.int8, device="cuda")
    rs = torch.empty(T, dtype=torch.int32, device="cuda")
    print("stage ln1", flush=True)
    off1 = b.rq_ln_quant(ctx, dev(x), dev(ln1["gamma_t"]), dev(ln1["beta_t"]), float(ln1["s"]), int(ln1["z"]), ba, q, norm_kind=cfg.norm,
                         eps=cfg.eps, rowsum=rs)
    assert_codes_close(q.cpu().numpy().astype(np.int64) + off1, t["a1"], "ln1")
    print("stage qkv", flush=True)
    A = dev((t["a1"] - off1).astype(np.int8))
    b.rq_rowsum_i8(ctx, A, rs)
    offs = [b.store_offset(ba, int(P[k])) for k in ("z_q", "z_k", "z_v")]
    out = torch.zeros((T, 3 * D), dtype=torch.int8, device="cuda")
    b.rq_qgemm(ctx, A, off1, int(ln1["z"]), float(ln1["s"]), lin_to_device(P["qkv"], bw), out_q=out, bits_o=ba,
               s_o=[float(P["s_q"]), float(P["s_k"]), float(P["s_v"])], z_o=[int(P["z_q"]), int(P["z_k"]), int(P["z_v"])], off_o=offs,
               seg_len=D, rowsum_a=rs)
    go = out.cpu().numpy().astype(np.int64)
    for i, k in enumerate(("qq", "qk", "qv")):
        assert_codes_close(go[:, i * D:(i + 1) * D] + offs[i], t[k], "qkv " + k)
    print("stage qk", flush=True)
    qkv = dev(np.concatenate([t["qq"] - offs[0], t["qk"] - offs[1], t["qv"] - offs[2]], axis=1).astype(np.int8))
    ld = (N + 15) // 16 * 16
    acc = torch.zeros((H, N, ld), dtype=torch.int32, device="cuda")
    b.rq_qk(ctx, qkv, 1, N, H, dh, 0, D, offs[0], int(P["z_q"]), offs[1], int(P["z_k"]), acc, ld, causal=True)
    m = np.tril(np.ones((N, N), bool))
    assert np.array_equal(acc.cpu().numpy()[:, :, :N][:, m], t["acc"][0][:, m])
    print("stage softmax", flush=True)
    accd = torch.zeros((H, N, ld), dtype=torch.int32, device="cuda")
    accd[:, :, :N] = torch.from_numpy(t["acc"][0]).cuda()
    codes = torch.zeros((H, N, ld), dtype=torch.uint8, device="cuda")
    scale = float(P["s_q"]) * float(P["s_k"]) / math.sqrt(dh)
    b.rq_softmax_log2_quant(ctx, accd, H, H, N, N, ld, scale, codes, bp, s_log=float(P["s_log"]), mask=b.MASK_CAUSAL)
    assert_codes_close(codes.cpu().numpy()[:, :, :N][:, m], t["codes"][0][:, m], "softmax codes")
    print("stage pv", flush=True)
    cp = torch.zeros((H, N, ld), dtype=torch.uint8, device="cuda")
    cp[:, :, :N] = torch.from_numpy(t["codes"][0]).cuda()
    offo = b.store_offset(ba, int(P["z_o"]))
    outq = torch.zeros((T, D), dtype=torch.int8, device="cuda")
    outf = torch.zeros((T, D), dtype=torch.float32, device="cuda")
    b.rq_attn_pv(ctx, cp, ld, qkv.data_ptr() + 2 * D, 3 * D, 1, H, N, N, dh, float(P["s_log"]), float(P["s_v"]), int(P["z_v"]), offs[2], bp,
                 mask=b.MASK_CAUSAL, out_f32=outf, out_q=outq, s_o=float(P["s_o"]), z_o=int(P["z_o"]), off_o=offo, bits_o=ba)
    assert_float_close(outf.cpu().numpy(), t["attn"], "pv", rtol=1e-5)
    assert_codes_close(outq.cpu().numpy().astype(np.int64) + offo, t["qo"], "pv codes")
    print("stage proj", flush=True)
    A = dev((t["qo"] - offo).astype(np.int8))
    b.rq_rowsum_i8(ctx, A, rs)
    xb = torch.zeros((T, D), dtype=torch.float32, device="cuda")
    b.rq_qgemm(ctx, A, offo, int(P["z_o"]), float(P["s_o"]), lin_to_device(P["proj"], bw), residual=dev(x), out_f32=xb, rowsum_a=rs)
    assert_float_close(xb.cpu().numpy(), t["xbar"], "proj")
    print("stage ln2", flush=True)
    xbar32 = t["xbar"].astype(np.float32)
    off2 = b.rq_ln_quant(ctx, dev(xbar32), dev(ln2["gamma_t"]), dev(ln2["beta_t"]), float(ln2["s"]), int(ln2["z"]), ba, q,
                         norm_kind=cfg.norm, eps=cfg.eps, rowsum=rs)
    assert_codes_close(q.cpu().numpy().astype(np.int64) + off2, t["a2"], "ln2")
    print("stage fc1", flush=True)
    A = dev((t["a2"] - off2).astype(np.int8))
    b.rq_rowsum_i8(ctx, A, rs)
    offh = b.store_offset(ba, int(P["z_h"]))
    hq = torch.zeros((T, Dm), dtype=torch.int8, device="cuda")
    b.rq_qgemm(ctx, A, off2, int(ln2["z"]), float(ln2["s"]), lin_to_device(P["fc1"], bw, Dm), act=b.ACT_SILU_GATED, out_q=hq, bits_o=ba,
               s_o=[float(P["s_h"])], z_o=[int(P["z_h"])], off_o=[offh], seg_len=Dm, rowsum_a=rs)
    assert_codes_close(hq.cpu().numpy().astype(np.int64) + offh, t["qh"], "fc1 codes")
    print("stage fc2", flush=True)
    A = dev((t["qh"] - offh).astype(np.int8))
    b.rq_rowsum_i8(ctx, A, rs)
    yo = torch.zeros((T, D), dtype=torch.float32, device="cuda")
    b.rq_qgemm(ctx, A, offh, int(P["z_h"]), float(P["s_h"]), lin_to_device(P["fc2"], bw), residual=dev(xbar32), out_f32=yo, rowsum_a=rs)
    assert_float_close(yo.cpu().numpy(), y_ref, "fc2")
    print("whole block", flush=True)
    blk = b.Block(ctx, cfg, block_to_device(P))
    xd = dev(x)
    yb = torch.zeros_like(xd)
    blk.forward(xd, yb, cfg.batch, cfg.seq)
    torch.cuda.synchronize()
    got_y = yb.cpu().numpy().astype(np.float64)
    ref = np.abs(y_ref).max()
    e = np.abs(got_y - y_ref).max(axis=1)
    print("  end to end: max|d| / max|ref| = %.3g, rows beyond 1e-3: %.3g, median row error %.3g"
          % (e.max() / ref, float(np.mean(e > 1e-3 * ref)), float(np.median(e)) / ref), flush=True)
    # ---- what the kernels left in the workspace: every code tensor of the pass ----
    lay = blk.layout(cfg.batch, cfg.seq)
    assert lay.codes_bytes >= H * N * lay.ld and lay.batch_chunk == 1
    inter = blk.intermediates(cfg.batch, cfg.seq)
    g_qkv = inter["qkv"].cpu().numpy().astype(np.int64)
    g_q, g_k, g_v = (g_qkv[:, i * D:(i + 1) * D] + offs[i] for i in range(3))
    g_codes = inter["codes"].cpu().numpy()[:, :, :N].astype(np.int64)
    g_o = inter["o"].cpu().numpy().astype(np.int64) + offo
    g_xbar = inter["xbar"].cpu().numpy()
    g_a2 = inter["a2"].cpu().numpy().astype(np.int64) + off2
    g_h = inter["hidden"].cpu().numpy().astype(np.int64) + offh
    flips = {k: int(np.count_nonzero(a != w)) for k, a, w in (("q", g_q, t["qq"]), ("k", g_k, t["qk"]), ("v", g_v, t["qv"]))}
    print("  Q / K / V codes that differ from the oracle's: %s of %d each" % (flips, T * D), flush=True)
    for k, a, w in (("q", g_q, t["qq"]), ("k", g_k, t["qk"]), ("v", g_v, t["qv"])):
        assert_codes_close(a, w, "block " + k)
    # ---- the oracle's stages fed with the codes the kernels produced (every code the GPU chose differently sits on a
    # rounding tie and is inside the 1e-4 budget; given the same codes, the floats must agree to 1e-3) ----
    attn = np.empty((T, D))
    code_flips = 0
    reached = np.zeros(T, bool)               # rows that a differing code upstream of the Softmax output can reach
    reached |= (g_q != t["qq"]).any(axis=1)
    for arr, w in ((g_k, t["qk"]), (g_v, t["qv"])):
        rows_kv = np.flatnonzero((arr != w).any(axis=1))
        if rows_kv.size:
            reached[rows_kv.min():] = True    # causal: a key / value row is seen by the queries after it
    for h in range(H):
        cs = slice(h * dh, (h + 1) * dh)
        L, _ = orc.attention_logits(g_q[:, cs], P["z_q"], P["s_q"], g_k[:, cs], P["z_k"], P["s_k"], dh, None, True)
        want_codes = orc.softmax_log_quant(L, P["s_log"], bp)
        d = np.abs(want_codes - g_codes[h])[m]
        assert d.max() <= 1
        code_flips += int(np.count_nonzero(d))
        reached |= ((g_codes[h] != t["codes"][0][h].astype(np.int64)) & m).any(axis=1)
        attn[:, cs] = orc.attn_pv(g_codes[h], g_v[:, cs], P["s_log"], P["s_v"], P["z_v"], True)
    print("  Softmax codes that differ from the oracle's on the GPU's own Q, K: %d of %d" % (code_flips, H * N * (N + 1) // 2), flush=True)
    assert code_flips <= 1e-4 * H * N * (N + 1) // 2
    assert_codes_close(g_o, orc.uniform_quant(attn, P["s_o"], P["z_o"], ba), "block attention output codes")
    xbar_w = orc.qlinear(g_o, P["s_o"], P["z_o"], P["proj"]) + x.astype(np.float64)
    assert_float_close(g_xbar, xbar_w, "block xbar")
    assert_codes_close(g_a2, orc.ln_quant(g_xbar.astype(np.float64), ln2["gamma_t"], ln2["beta_t"], ln2["s"], ln2["z"], ba, cfg.eps, cfg.norm),
                       "block ln2 codes")
    hid_w = orc.mlp_activation(orc.qlinear(g_a2, ln2["s"], ln2["z"], P["fc1"]), cfg.act, Dm)
    assert_codes_close(g_h, orc.uniform_quant(hid_w, P["s_h"], P["z_h"], ba), "block hidden codes")
    y_w = orc.qlinear(g_h, P["s_h"], P["z_h"], P["fc2"]) + g_xbar.astype(np.float64)
    assert_float_close(got_y, y_w, "block y from the GPU's own codes")
    # ---- and end to end against the oracle's own pass.  Codes downstream of the Softmax (attention output, LayerNorm-2,
    # MLP hidden) are taken from float32 tensors on the GPU and from float64 ones in the oracle, so a few sit on the other
    # side of a rounding tie (all inside the budget, checked above); in the outlier channels of this workload one such
    # LayerNorm-2 code moves its row by ~1e-3 of the block's largest output.  Rows that hold no differing code at any stage
    # must meet the stated bar; the others are explained by their codes (the chain above) and stay within a few steps. ----
    touched = reached.copy()
    stage_flips = {}
    for k, a, w in (("attention output", g_o, t["qo"]), ("ln2", g_a2, t["a2"]), ("hidden", g_h, t["qh"])):
        rows_k = (a != w).any(axis=1)
        stage_flips[k] = (int(np.count_nonzero(a != w)), int(rows_k.sum()))
        touched |= rows_k
    print("  rows reached by a differing code upstream of P.V: %d of %d; differing codes (count, rows): %s; rows with none anywhere: %d"
          % (int(reached.sum()), T, stage_flips, int((~touched).sum())), flush=True)
    assert reached.mean() <= 0.1
    assert (~touched).sum() >= T // 4
    assert e[~touched].max() <= 1e-3 * ref                  # every row no differing code reached: the stated bar
    if not touched.any():
        assert e.max() <= 1e-3 * ref
    assert e.max() <= 5e-3 * ref and float(np.mean(e > 1e-3 * ref)) <= 0.01
    assert np.median(e) <= 1e-4 * ref

#!/usr/bin/env python3
"""Benchmark of the reparameterized quantized transformer block on one MI355X.

A step is one rq_block_forward over one synthetic batch (all kernels of the hot path: LN-quant, QKV GEMM,
Q.K^T, softmax-log2, P.V, proj GEMM, LN-quant, FC1 GEMM, FC2 GEMM), inputs and parameters resident in HBM.
Prints ONE JSON line: tokens/s, the roofline of the dominant kernel (measured live with HIP events on the
library's stream in a second, instrumented pass of the same length) and the CPU oracle timed on a bounded
sample of the same workload on the host cores.
"""
from __future__ import annotations

import argparse
import dataclasses
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0     # MI355X dense int8 MFMA, TOP/s
PEAK_FP64_TFLOPS = 78.6       # MI355X vector float64
PEAK_HBM_GBS = 8000.0       # MI355X HBM3E, GB/s


def algorithmic_work(cfg, ld):
    """Per-step algorithmic ops / bytes of every kernel family (bytes and ops a perfect implementation must move / do)."""
    T, D, Dm, H, N = cfg.tokens, cfg.D, cfg.Dm, cfg.H, cfg.seq
    G = cfg.batch * H
    dh = D // H
    n1 = 2 * Dm if cfg.act != 0 else Dm
    wb = cfg.bits_w / 8.0 if cfg.bits_w == 4 else 1.0
    causal = cfg.mask != 0
    nn = N * (N + 1) // 2 if causal else N * N
    gemm = {
        "qkv": (T, 3 * D, D, 1), "proj": (T, D, D, 4), "fc1": (T, n1, D, 1), "fc2": (T, D, Dm, 4),
    }
    w = {}
    for k, (M, Nn, K, ob) in gemm.items():
        n_out = Nn // 2 if (k == "fc1" and cfg.act != 0) else Nn
        w[k] = dict(ops=2.0 * M * Nn * K, bytes=M * K + Nn * K * wb + M * n_out * ob + (M * n_out * 4 if ob == 4 else 0))
    w["ln1"] = w["ln2"] = dict(ops=0.0, bytes=5.0 * T * D)
    w["qk"] = dict(ops=2.0 * G * nn * dh, bytes=G * (2 * N * dh + 4.0 * nn))
    w["softmax"] = dict(ops=0.0, bytes=5.0 * G * nn)
    w["pv"] = dict(ops=2.0 * G * nn * dh, bytes=G * (1.0 * nn + N * dh) + T * D)
    return w


def read_traffic(path):
    """HBM bytes per GEMM launch from the committed rocprofv3 --pmc summary (FETCH_SIZE + WRITE_SIZE), or None."""
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch"):
                return float(line.split("=")[1].split()[0])
    except OSError:
        pass
    return None


def standalone_row_kernels(rq, ctx, cfg, torch):
    """rq_ln_quant and rq_softmax_log2_quant alone at this workload's shapes, HIP events on the library's stream.
    The inputs rotate over buffer sets larger than the 256 MB last-level cache, so the bytes come from HBM."""
    out = {}
    T, D, G, N = cfg.tokens, cfg.D, cfg.batch * cfg.H, cfg.seq
    ld = (N + 15) // 16 * 16

    def timed(calls, reps):
        for c in calls:
            c()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            for c in calls:
                c()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (reps * len(calls))

    nset = max(2, int(300e6 // (T * D * 4)) + 1)
    xs = [torch.randn(T, D, device="cuda") for _ in range(nset)]
    gam, bet = torch.ones(D, device="cuda"), torch.zeros(D, device="cuda")
    q = torch.empty((T, D), dtype=torch.int8, device="cuda")
    ms = timed([(lambda x=x: rq.rq_ln_quant(ctx, x, gam, bet, 0.4, 2 ** cfg.bits_a // 2, cfg.bits_a, q)) for x in xs], 10)
    gbs = 5.0 * T * D / (ms * 1e-3) / 1e9
    out["ln_quant"] = dict(achieved=gbs, peak=PEAK_HBM_GBS, unit="GB/s", frac=gbs / PEAK_HBM_GBS, ms_per_launch=ms,
                           bytes_per_launch=5.0 * T * D, buffers=nset)
    del xs
    if cfg.mask == 0 and G * N * ld * 4 <= 1 << 30:
        nset = max(2, int(300e6 // (G * N * ld * 4)) + 1)
        accs = [torch.randint(-3000, 3000, (G, N, ld), dtype=torch.int32, device="cuda") for _ in range(nset)]
        codes = torch.empty((G, N, ld), dtype=torch.uint8, device="cuda")
        scale = 0.0625 * 0.0625 / (cfg.D // cfg.H) ** 0.5
        ms = timed([(lambda a=a: rq.rq_softmax_log2_quant(ctx, a, G, cfg.H, N, N, ld, scale, codes, cfg.bits_p)) for a in accs], 10)
        gbs = 5.0 * G * N * N / (ms * 1e-3) / 1e9
        out["softmax_log2_quant"] = dict(achieved=gbs, peak=PEAK_HBM_GBS, unit="GB/s", frac=gbs / PEAK_HBM_GBS, ms_per_launch=ms,
                                         bytes_per_launch=5.0 * G * N * N, buffers=nset)
    return out


DUAL_CLIP_FLOPS_PER_ELEMENT_PASS = 17      # mul, round, 7 add/sub, 2 compare, min, max, mul, 2 fma (4)


def copy_reference(torch):
    """What a kernel with nothing but memory traffic reaches on this machine: plain device-to-device copies (torch's copy_),
    1 GiB (served from HBM) and 128 MiB (partly from the 256 MB last-level cache).  Context for the HBM-bound kernels'
    fractions of the published peak; not a kernel of this library."""
    out = {}
    for name, n, reps in (("copy_1GiB", 1 << 30, 10), ("copy_128MiB", 128 << 20, 30)):
        a = torch.empty(n // 4, dtype=torch.float32, device="cuda").normal_()
        b = torch.empty_like(a)
        for _ in range(3):
            b.copy_(a)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            b.copy_(a)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        out[name] = dict(ms=ms, achieved=2 * n / (ms * 1e-3) / 1e9, unit="GB/s", frac_of_peak=2 * n / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS)
        del a, b
    return out


def bench_dual_clip(args, cfg, rq, synth, np, torch):
    """One step = learning the clipping factors of one LayerNorm activation [T, D] (100 Adam iterations)."""
    iters, lr, alpha0 = 100, 0.01, 4.0
    torch.cuda.set_device(0)
    ctx = rq.Context(0)
    raw = synth.make_block(cfg, args.config, 0)
    x = torch.from_numpy(raw["x"]).cuda()
    gamma, beta = torch.from_numpy(raw["ln1_gamma"]).cuda(), torch.from_numpy(raw["ln1_beta"]).cuda()
    run = lambda: rq.rq_dual_clip_learn(ctx, x, cfg.bits_a, gamma=gamma, beta=beta, norm_kind=cfg.norm, eps=cfg.eps, iters=iters,
                                        lr=lr, alpha0=alpha0)
    steps, warmup = min(args.steps, 20), min(args.warmup, 3)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    flops = DUAL_CLIP_FLOPS_PER_ELEMENT_PASS * cfg.tokens * cfg.D * (iters + 1)
    achieved = flops / sec / 1e12
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import dual_clip_oracle as dco
        from oracle import repquant_oracle as orc
        Xp = orc.layernorm(raw["x"].astype(np.float64), raw["ln1_gamma"].astype(np.float64), raw["ln1_beta"].astype(np.float64),
                           cfg.eps, cfg.norm)
        nch = min(cfg.D, 384)
        c0 = time.perf_counter()
        dco.learn(Xp[:, :nch], cfg.bits_a, iters=iters, lr=lr, alpha0=alpha0)
        c1 = time.perf_counter()
        cpu = dict(value=(c1 - c0) * cfg.D / nch, unit="s per layer", cores=torch.get_num_threads(), kind="oracle",
                   sample="%d of %d channels, all %d tokens, %d iterations: %.1f s, scaled by the channel count (channels are "
                          "independent problems)" % (nch, cfg.D, cfg.tokens, iters, c1 - c0))
    out = dict(metric="dual-clipping learner, seconds per layer on 1 MI355X", value=sec, unit="s per layer", n_gpus=1, steps=steps,
               warmup=warmup, ms_per_step=sec * 1e3, higher_is_better=False, scaling="weak", vs_baseline=None, dtype="f64",
               data="synthetic",
               config=dict(workload=cfg.name + " LayerNorm-1 activation", tokens=cfg.tokens, hidden=cfg.D, bits_a=cfg.bits_a,
                           iterations=iters, lr=lr, alpha0=alpha0),
               roofline=dict(bound="alu", kernel="dual_clip_kernel", achieved=achieved, peak=PEAK_FP64_TFLOPS, unit="TFLOP/s",
                             frac=achieved / PEAK_FP64_TFLOPS, traffic=None, flops_per_launch=flops),
               cpu_baseline=cpu)
    print(json.dumps(out))


def bench_gptq(args, cfg, rq, synth, np, torch):
    """One step = GPTQ of the QKV weight matrix [3D, D] against the block's LayerNorm-1 codes [T, D]."""
    torch.cuda.set_device(0)
    ctx = rq.Context(0)
    g = synth.rng_for(args.config, 7)
    N, K, T = 3 * cfg.D, cfg.D, cfg.tokens
    W = (g.standard_normal((N, K)) * 0.02).astype(np.float32)
    qmax = 2 ** cfg.bits_a - 1
    z_a = qmax // 2 + 1
    F = g.standard_normal((T, 8))
    codes = np.clip(np.rint((F @ g.standard_normal((8, K)) * 0.5 + g.standard_normal((T, K))) * (qmax / 8.0)) + z_a, 0, qmax)
    off = z_a if cfg.bits_a < 8 else 128
    Wd, Ad = torch.from_numpy(W).cuda(), torch.from_numpy((codes - off).astype(np.int8)).cuda()
    run = lambda: rq.rq_gptq_quant_pack(ctx, Wd, None, cfg.bits_w, Ad, off, z_a)
    steps, warmup = min(args.steps, 20), min(args.warmup, 3)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        run()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    # float64 work: Cholesky K^3/3, triangular inverse K^3/3, sweep N K^2 (in-block and lazy updates together)
    flops = 2.0 * K ** 3 / 3.0 + float(N) * K * K
    achieved = flops / sec / 1e12
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import gptq_oracle as gq
        c0 = time.perf_counter()
        gq.gptq(W, codes.astype(np.int64) - z_a, cfg.bits_w)
        c1 = time.perf_counter()
        cpu = dict(value=c1 - c0, unit="s per layer", cores=torch.get_num_threads(), kind="oracle",
                   sample="the whole layer (%d x %d weights, %d tokens), elimination-form float64 numpy oracle" % (N, K, T))
    out = dict(metric="GPTQ of one linear layer, seconds on 1 MI355X", value=sec, unit="s per layer", n_gpus=1, steps=steps,
               warmup=warmup, ms_per_step=sec * 1e3, higher_is_better=False, scaling="weak", vs_baseline=None, dtype="f64",
               data="synthetic", config=dict(workload=cfg.name + " QKV weights", N=N, K=K, tokens=T, bits_w=cfg.bits_w, bits_a=cfg.bits_a),
               roofline=dict(bound="alu", kernel="rq_gptq_quant_pack (all kernels of the call)", achieved=achieved, peak=PEAK_FP64_TFLOPS,
                             unit="TFLOP/s", frac=achieved / PEAK_FP64_TFLOPS, traffic=None, flops_per_launch=flops),
               cpu_baseline=cpu)
    print(json.dumps(out))


def bench_gemm(args, rq, np, torch):
    """One step = one large quantized linear layer, 8192 x 8192 x 8192: int8 activation codes times packed 4-bit weights
    on the int8 matrix cores, re-quantized to int8 codes in the epilogue (rq_qgemm, weight mode)."""
    torch.cuda.set_device(0)
    ctx = rq.Context(0)
    M = N = 8192
    K = args.gemm_k
    g = torch.Generator(device="cuda")
    g.manual_seed(3)
    A = torch.randint(-8, 8, (M, K), dtype=torch.int8, device="cuda", generator=g)
    W = torch.randn((N, K), device="cuda", generator=g) * 0.02
    fmt = rq.W_I8_BAKED if args.wfmt == "i8" else rq.W_U4
    lin = rq.rq_weight_quant_pack(ctx, W, torch.zeros(N, device="cuda"), 4, fmt=fmt)
    out = torch.empty((M, N), dtype=torch.int8, device="cuda")
    rs = torch.empty(M, dtype=torch.int32, device="cuda")
    rq.rq_rowsum_i8(ctx, A, rs)      # with the row sums at hand the kernel multiplies the raw 4-bit codes
    rq.set_gemm_tile(ctx, args.tile)
    run = lambda: rq.rq_qgemm(ctx, A, 8, 8, 0.01, lin, rowsum_a=rs, out_q=out, bits_o=4, s_o=[0.1], z_o=[8], off_o=[8], seg_len=N)
    steps, warmup = min(args.steps, 20), min(args.warmup, 3)
    for _ in range(warmup):
        run()
    torch.cuda.synchronize()
    s, e = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    s.record()
    for _ in range(steps):
        run()
    e.record()
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / steps
    kernel_ms = s.elapsed_time(e) / steps
    ops = 2.0 * M * N * K
    achieved = ops / (kernel_ms * 1e-3) / 1e12
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import repquant_oracle as orc
        rows = M       # the whole product, against a weight matrix of the same shape
        a = A[:rows].cpu().numpy().astype(np.int64)
        wq = np.random.default_rng(3).integers(-8, 8, size=(N, K), dtype=np.int64)
        c0 = time.perf_counter()
        orc.int_matmul_nt(a, wq)
        c1 = time.perf_counter()
        cpu = dict(value=2.0 * rows * N * K / (c1 - c0) / 1e12, unit="TOP/s", cores=torch.get_num_threads(), kind="oracle",
                   sample="%d of %d output rows: the oracle's exact integer product (float64 BLAS on integers) against %d x %d weights; %.1f s"
                          % (rows, M, N, K, c1 - c0))
    out_d = dict(metric="quantized GEMM int8 TOP/s on 1 MI355X", value=ops / sec / 1e12, unit="TOP/s", n_gpus=1, steps=steps, warmup=warmup,
                 ms_per_step=sec * 1e3, higher_is_better=True, scaling="weak", vs_baseline=None, dtype="int8", data="synthetic",
                 config=dict(workload="qgemm_w4a8_8192" if K == 8192 else "qgemm_w4a8_8192x8192x%d" % K, M=M, N=N, K=K, bits_w=4, weight_storage=args.wfmt,
                             output="re-quantized int8 codes"),
                 roofline=dict(bound="mfma", kernel="qgemm_pipe_kernel (256 x 256 tiles)", achieved=achieved, peak=PEAK_INT8_TOPS, unit="TOP/s",
                               frac=achieved / PEAK_INT8_TOPS, traffic=None, avg_launch_ms=kernel_ms, ops_per_launch=ops),
                 cpu_baseline=cpu)
    print(json.dumps(out_d))


GEMMS = ("qkv", "proj", "fc1", "fc2")


def run_block(args, cfg_id, cfg, ctx, rq, synth, np, torch, full):
    """Times rq_block_forward on one workload; returns the JSON record.  full=False: the timed pass and the instrumented
    pass only (no stand-alone row kernels, no CPU leg)."""
    steps, warmup = (args.steps, args.warmup) if full else (min(args.steps, 20), min(args.warmup, 5))
    raw = synth.make_block(cfg, cfg_id, 0)
    x = torch.from_numpy(raw["x"]).cuda()
    rawd = {k: (None if v is None else torch.from_numpy(v).cuda()) for k, v in raw.items() if k != "x"}
    blk = rq.calibrate_block(ctx, cfg, rawd, x, cfg.batch, cfg.seq)       # untimed preparation, on the GPU
    del rawd, raw
    if args.chunk_mb:
        blk.bp.attn_chunk_bytes = args.chunk_mb << 20
    y = torch.empty_like(x)

    for _ in range(warmup):
        blk.forward(x, y, cfg.batch, cfg.seq)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        blk.forward(x, y, cfg.batch, cfg.seq)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / steps
    tokens_per_s = cfg.tokens / (ms_per_step * 1e-3)

    # second pass of the same length with HIP events around every kernel launch (on the library's stream)
    rq.profile_enable(ctx, True)
    rq.profile_reset(ctx)
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    for _ in range(steps):
        blk.forward(x, y, cfg.batch, cfg.seq)
    prof = rq.profile_read(ctx)
    t3 = time.perf_counter()
    rq.profile_enable(ctx, False)
    ld = (cfg.seq + 15) // 16 * 16
    work = algorithmic_work(cfg, ld)
    kern = {}
    for name, (ms, n) in prof.items():
        if n == 0 or name not in work:
            continue
        per_step_ms = ms / steps
        kern[name] = dict(ms_per_step=per_step_ms, launches_per_step=n / steps,
                          tops=work[name]["ops"] / (per_step_ms * 1e-3) / 1e12,
                          gbs=work[name]["bytes"] / (per_step_ms * 1e-3) / 1e9)
    # dominant kernel: the weight-mode int8 MFMA GEMM (four launches per step, one kernel family).  Each launch against the
    # roofline that bounds IT: max(ops / int8 peak, algorithmic bytes / HBM peak).
    launches = {}
    for k in GEMMS:
        ops, nbytes, ms = work[k]["ops"], work[k]["bytes"], kern[k]["ms_per_step"]
        t_mfma, t_hbm = ops / (PEAK_INT8_TOPS * 1e12) * 1e3, nbytes / (PEAK_HBM_GBS * 1e9) * 1e3
        launches[k] = dict(ms=ms, ops=ops, bytes=nbytes, achieved_tops=kern[k]["tops"], frac_of_int8_peak=kern[k]["tops"] / PEAK_INT8_TOPS,
                           achieved_gbs=kern[k]["gbs"], bound="mfma" if t_mfma >= t_hbm else "hbm", roofline_ms=max(t_mfma, t_hbm),
                           frac_of_own_roofline=max(t_mfma, t_hbm) / ms)
    gemm_ms = sum(kern[k]["ms_per_step"] for k in GEMMS)
    gemm_ops = sum(work[k]["ops"] for k in GEMMS)
    gemm_bytes = sum(work[k]["bytes"] for k in GEMMS)
    achieved = gemm_ops / (gemm_ms * 1e-3) / 1e12
    agg_bound = "mfma" if gemm_ops / (PEAK_INT8_TOPS * 1e12) >= gemm_bytes / (PEAK_HBM_GBS * 1e9) else "hbm"
    roofline = dict(bound=agg_bound, kernel="qgemm_pipe_kernel (qkv+proj+fc1+fc2; per launch: gemm_launches)", achieved=achieved,
                    peak=PEAK_INT8_TOPS, unit="TOP/s", frac=achieved / PEAK_INT8_TOPS, traffic=None,
                    avg_launch_ms=gemm_ms / 4.0, ops_per_launch=gemm_ops / 4.0, bytes_per_launch=gemm_bytes / 4.0,
                    share_of_step=gemm_ms / sum(v["ms_per_step"] for v in kern.values()))
    roofline["traffic"] = read_traffic(os.path.join(ROOT, "profiles", "qgemm_%s_hbm_traffic.txt" % cfg.name))
    hbm = {}
    for k in ("ln1", "ln2", "softmax"):
        if k in kern:
            hbm[k + "_in_block"] = dict(achieved=kern[k]["gbs"], peak=PEAK_HBM_GBS, unit="GB/s", frac=kern[k]["gbs"] / PEAK_HBM_GBS,
                                        ms_per_launch=kern[k]["ms_per_step"] / kern[k]["launches_per_step"])
    if full:
        hbm.update(standalone_row_kernels(rq, ctx, cfg, torch))

    cpu = None
    if full and not args.no_cpu_baseline:
        from oracle import repquant_oracle as orc
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count() or 1
        cal_cfg = cfg.with_batch(min(cfg.batch, 4))
        run_cfg = cfg.with_batch(min(cfg.batch, 64 if cfg.seq <= 512 else 1))
        raw_c = synth.make_block(cal_cfg, cfg_id, 1)
        P = orc.calibrate_block(raw_c, dataclasses.asdict(cal_cfg))
        P["cfg"] = dataclasses.asdict(run_cfg)
        xs = synth.make_block(run_cfg, cfg_id, 2)["x"]
        passes, c0 = 0, time.perf_counter()
        while passes < 40 and time.perf_counter() - c0 < 12.0:   # whole passes, about 12 s of host work
            orc.block_forward(P, xs)
            passes += 1
        c1 = time.perf_counter()
        cpu = dict(value=passes * run_cfg.tokens / (c1 - c0), unit="tokens/s", cores=cores, kind="oracle",
                   sample="%d forward passes over %d of %d sequences of the same workload (%d tokens each pass; tokens/s does not "
                          "depend on the number of sequences, they never interact), float64 numpy oracle calibrated on %d sequences; "
                          "%.1f s" % (passes, run_cfg.batch, cfg.batch, run_cfg.tokens, cal_cfg.batch, c1 - c0))

    del blk
    torch.cuda.empty_cache()
    return dict(metric="quantized-block tokens/s on 1 MI355X", value=tokens_per_s, unit="tokens/s", n_gpus=1,
                steps=steps, warmup=warmup, ms_per_step=ms_per_step, higher_is_better=True, scaling="weak",
                vs_baseline=None, dtype="int8", data="synthetic",
                config=dict(workload=cfg.name, batch=cfg.batch, seq=cfg.seq, hidden=cfg.D, heads=cfg.H, mlp=cfg.Dm,
                            bits_w=cfg.bits_w, bits_a=cfg.bits_a, bits_softmax=cfg.bits_p, tokens=cfg.tokens,
                            streams=("two halves of the batch side by side on two streams (library default at this size); the "
                                     "instrumented pass behind kernels_ms_per_step and roofline runs on one"
                                     if cfg.tokens * cfg.D >= (16 << 20) and cfg.batch >= 2 and cfg.seq <= 288 and args.streams != 1 else "one")),
                roofline=roofline, gemm_launches=launches, hbm_kernels=hbm,
                kernels_ms_per_step={k: round(v["ms_per_step"], 5) for k, v in kern.items()},
                ms_per_step_instrumented=(t3 - t2) * 1e3 / steps, cpu_baseline=cpu)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=4,
                    help="index into the synthetic workloads; default 4: CLIP ViT-L/14 image tower W4/A4, 128 x 257 tokens, the "
                         "largest single-GPU workload (862 GOP per step)")
    ap.add_argument("--also", default="3,1", help="further workloads timed briefly in the same run (comma-separated; '' for none)")
    ap.add_argument("--batch", type=int, default=0, help="override the batch of the workload")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--chunk-mb", type=int, default=0)
    ap.add_argument("--tile", type=int, default=0)
    ap.add_argument("--streams", type=int, default=2, choices=[1, 2, 3],
                    help="rq_set_block_streams: 1 = one stream, 2 = the library's default (large batches run as two halves side by side), 3 = always two")
    ap.add_argument("--gemm-k", type=int, default=8192, help="gemm workload: inner dimension (a multiple of 64)")
    ap.add_argument("--wfmt", default="u4", choices=["u4", "i8"],
                    help="gemm workload: storage of the 4-bit weight codes -- u4: two codes per byte; i8: one int8 per code "
                         "with the zero-point already subtracted (twice the weight bytes, no unpacking in the kernel)")
    ap.add_argument("--copy-probe", action="store_true", help="append three 256 MiB elementwise copies (counter calibration)")
    ap.add_argument("--workload", default="block", choices=["block", "dual_clip", "gptq", "gemm"],
                    help="block: the quantized block forward (the headline metric); dual_clip: the calibration-side learner of "
                         "the per-channel clipping factors on the same activations; gptq: GPTQ of the QKV weights against them; "
                         "gemm: one large quantized linear layer (8192^3, packed 4-bit weights)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (batch items never interact, so more GPUs "
              "would each take a slice of the batch with the same folded weights)." % args.gpus, file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2402_05628_amd import binding as rq
    from paper_2402_05628_amd import synth

    cfg = synth.CONFIGS[args.config]
    if args.batch:
        cfg = cfg.with_batch(args.batch)
    if args.workload == "dual_clip":
        return bench_dual_clip(args, cfg, rq, synth, np, torch)
    if args.workload == "gptq":
        return bench_gptq(args, cfg, rq, synth, np, torch)
    if args.workload == "gemm":
        return bench_gemm(args, rq, np, torch)
    torch.cuda.set_device(0)
    ctx = rq.Context(0)
    if args.tile:
        rq.set_gemm_tile(ctx, args.tile)
    if args.streams != 2:
        rq.set_block_streams(ctx, args.streams)
    out = run_block(args, args.config, cfg, ctx, rq, synth, np, torch, full=True)
    # the other large single-GPU workloads in the same run (shorter, no stand-alone kernels, no CPU leg): context for the
    # headline line, each with its own per-launch GEMM figures
    others = {}
    for c in [int(v) for v in args.also.split(",") if v.strip()]:
        if c != args.config and not args.batch:
            o = run_block(args, c, synth.CONFIGS[c], ctx, rq, synth, np, torch, full=False)
            others[o["config"]["workload"]] = dict(ms_per_step=o["ms_per_step"], tokens_per_s=o["value"], tokens=o["config"]["tokens"],
                                                   gemm_frac_of_int8_peak=o["roofline"]["frac"], gemm_launches=o["gemm_launches"],
                                                   kernels_ms_per_step=o["kernels_ms_per_step"])
    if others:
        out["other_workloads"] = others
    out["hbm_copy_reference"] = copy_reference(torch)
    print(json.dumps(out))
    if args.copy_probe:
        # a plain device copy of known size (256 MiB read + 256 MiB written): scales the HBM byte counters of a --pmc run
        a_ = torch.empty(64 << 20, dtype=torch.float32, device="cuda").normal_()
        b_ = torch.empty_like(a_)
        for _ in range(3):
            torch.add(a_, 1.0, out=b_)
        torch.cuda.synchronize()


if __name__ == "__main__":
    main()

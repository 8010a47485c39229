"""CPU oracle for the RepQuant inference path -- TEST INFRASTRUCTURE ONLY.

Plain, slow, float64 numpy.  Nothing here is tuned, blocked or fused; every
function restates one passage of the paper (arXiv 2402.05628) so that it can be
checked against the text by eye.  Only tests/, __graft_entry__.smoke() and
bench.py's cpu_baseline leg may import this module; the product (the HIP
library and its Python binding) never does, and this module imports nothing
from the product.

Two tiers:

* "definition" tier (names ending in `_channelwise` / `_sqrt2`): the
  quantizers the paper uses in the *quantization process* -- channel-wise
  uniform quantization of LayerNorm activations, log-sqrt2 quantization of
  Softmax activations -- written as their plain definitions, no folding and no
  shifts.
* "reparameterized" tier: what runs at inference after scale
  reparameterization (Section "Scale Reparameterization"): layer-wise
  quantization with folded LayerNorm affine / next-layer weights, and log2-form
  quantization with a parity-selected scale.  The HIP path is compared to this
  tier; the definition tier pins it (the paper states the two are equal).

Conventions the paper leaves open:
  * rounding is round-half-to-even (numpy rint);
  * variance is the population variance; eps is a parameter;
  * z~ = rint(mean(z)) so that r2 = z - z~ is an integer vector;
  * the attention scale is 1/sqrt(d_head);
  * a Softmax value <= 0 takes the largest code; masked positions take no
    part in P.V;
  * every code, including the saturated one, dequantizes by the printed
    formula; the other reading of the saturated code (the paper is silent: it
    collects every probability below the grid, so it may be meant as "no mass")
    is the option `zero_at_max`, under which the largest code dequantizes to
    exactly 0 and every other code is unchanged;
  * stored scales are float32 numbers; all arithmetic on them is float64.

Parity unpinned by the paper (conventions fixed here, not checked against a
printed value): tie rule, eps, static min/max calibration of the non-LayerNorm
activations (the paper says "Percentile" without a value), erf-form GELU.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf as _erf

F64 = np.float64
SQRT2 = math.sqrt(2.0)

NORM_LAYERNORM = 0
NORM_RMSNORM = 1
ACT_GELU = 0
ACT_SILU_GATED = 1
MASK_NONE = 0
MASK_CAUSAL = 1


# --------------------------------------------------------------------------
# Section "Efficient quantizers"
# --------------------------------------------------------------------------
def qparams_from_bounds(lo, hi, bits):
    """Scale and zero-point from lower/upper bounds (Eq. for s and z).

    s = (x_up - x_low) / (2^b - 1),  z = round(-x_low / s).
    """
    lo = np.asarray(lo, dtype=F64)
    hi = np.asarray(hi, dtype=F64)
    s = (hi - lo) / (2 ** bits - 1)
    z = np.rint(-lo / s)
    return s, z.astype(np.int64)


def uniform_quant(x, s, z, bits):
    """Uniform quantizer: clip(round(x / s) + z, 0, 2^b - 1)."""
    x = np.asarray(x, dtype=F64)
    q = np.rint(x / np.asarray(s, dtype=F64)) + np.asarray(z, dtype=F64)
    return np.clip(q, 0, 2 ** bits - 1).astype(np.int64)


def uniform_dequant(q, s, z):
    """Uniform de-quantizer: s * (q - z)."""
    return np.asarray(s, dtype=F64) * (np.asarray(q, dtype=F64) - np.asarray(z, dtype=F64))


def log2_quant(x, s, bits):
    """log2 quantizer: clip(round(-log2(x / s)), 0, 2^b - 1); x <= 0 takes the largest code."""
    x = np.asarray(x, dtype=F64)
    qmax = 2 ** bits - 1
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.rint(-np.log2(x / F64(s)))
    q = np.where(x > 0, q, qmax)
    return np.clip(q, 0, qmax).astype(np.int64)


def log2_dequant(q, s):
    """log2 de-quantizer: s * 2^(-q)."""
    return F64(s) * np.exp2(-np.asarray(q, dtype=F64))


# --------------------------------------------------------------------------
# Section "Scale reparameterization for Softmax activations"
# --------------------------------------------------------------------------
def logsqrt2_quant(A, s, bits):
    """log-sqrt2 quantizer, first line of Eq. (3.3-1): clip(round(-log_sqrt2(A / s)), 0, 2^b - 1)."""
    A = np.asarray(A, dtype=F64)
    qmax = 2 ** bits - 1
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.rint(-np.log(A / F64(s)) / math.log(SQRT2))
    q = np.where(A > 0, q, qmax)
    return np.clip(q, 0, qmax).astype(np.int64)


def logsqrt2_quant_base2(A, s, bits):
    """Same quantizer after the change of base, second line of Eq. (3.3-1):
    clip(round(-2 * log2(A / s)), 0, 2^b - 1)."""
    A = np.asarray(A, dtype=F64)
    qmax = 2 ** bits - 1
    with np.errstate(divide="ignore", invalid="ignore"):
        q = np.rint(-2.0 * np.log2(A / F64(s)))
    q = np.where(A > 0, q, qmax)
    return np.clip(q, 0, qmax).astype(np.int64)


def logsqrt2_dequant(q, s, bits=None, zero_at_max=False):
    """log-sqrt2 de-quantizer, the definition: s * sqrt2^(-q).
    zero_at_max (needs bits): the saturated code 2^bits - 1 de-quantizes to 0 instead."""
    q = np.asarray(q)
    out = F64(s) * np.power(SQRT2, -q.astype(F64))
    if zero_at_max:
        out = np.where(q == 2 ** bits - 1, 0.0, out)
    return out


def parity_scale(q, s):
    """Reparameterized scale, Eq. (3.3-2): s~ = s * [1(q) * (sqrt2 - 1) + 1], 1(q) = parity of q."""
    q = np.asarray(q, dtype=np.int64)
    return F64(s) * ((q & 1).astype(F64) * (SQRT2 - 1.0) + 1.0)


def logsqrt2_dequant_shift(q, s, bits=None, zero_at_max=False):
    """De-quantizer in shift form (last line of the case analysis before Eq. (3.3-2)):
    s~(q) * 2^floor(-q / 2): an integer power of two times a scale picked by the code's parity.
    zero_at_max (needs bits): the saturated code 2^bits - 1 de-quantizes to 0 instead."""
    q = np.asarray(q, dtype=np.int64)
    shift = np.floor(-q.astype(F64) / 2.0)
    out = parity_scale(q, s) * np.exp2(shift)
    if zero_at_max:
        out = np.where(q == 2 ** bits - 1, 0.0, out)
    return out


# --------------------------------------------------------------------------
# Section "Scale reparameterization for LayerNorm activations"
# --------------------------------------------------------------------------
def layernorm(X, gamma, beta, eps, kind=NORM_LAYERNORM):
    """LayerNorm over the hidden dimension of each token (Eq. for X'_{n,:}).

    kind == NORM_RMSNORM drops the mean: x / sqrt(mean(x^2) + eps) * gamma + beta.
    """
    X = np.asarray(X, dtype=F64)
    gamma = np.asarray(gamma, dtype=F64)
    beta = np.asarray(beta, dtype=F64)
    if kind == NORM_LAYERNORM:
        mu = X.mean(axis=-1, keepdims=True)
        var = ((X - mu) ** 2).mean(axis=-1, keepdims=True)
        xhat = (X - mu) / np.sqrt(var + eps)
    else:
        ms = (X ** 2).mean(axis=-1, keepdims=True)
        xhat = X / np.sqrt(ms + eps)
    return xhat * gamma + beta


def channel_bounds(Xp, clip_up=None, clip_lo=None):
    """Per-channel bounds of the LayerNorm activation; with dual clipping the
    channel extremes are multiplied by contraction factors in [0, 1]
    (Eqs. for X'_up and X'_low; the factors are Sigmoid(alpha) there)."""
    Xp = np.asarray(Xp, dtype=F64)
    up = Xp.max(axis=0)
    lo = Xp.min(axis=0)
    if clip_up is not None:
        up = up * np.asarray(clip_up, dtype=F64)
    if clip_lo is not None:
        lo = lo * np.asarray(clip_lo, dtype=F64)
    return lo, up


def channel_percentile_bounds(Xp, q_lo, q_hi):
    """Per-channel percentile bounds of X' [T, D] (Section "Implementation details": "the default calibration strategy
    is Percentile"; the paper gives no value, so the two fractions q_lo < q_hi in [0, 1] are parameters).  The q-th
    fraction of n sorted values v_0 <= ... <= v_{n-1} sits at h = q (n - 1) and is interpolated linearly between
    v_floor(h) and v_floor(h)+1 -- numpy's default definition, used here as the library routine it is."""
    Xp = np.asarray(Xp, dtype=F64)
    lo = np.percentile(Xp, 100.0 * q_lo, axis=0)
    hi = np.percentile(Xp, 100.0 * q_hi, axis=0)
    return lo, hi


def ln_quant_channelwise(X, gamma, beta, s_ch, z_ch, bits, eps, kind=NORM_LAYERNORM):
    """Definition tier: LayerNorm, then channel-wise uniform quantization with s, z in R^D, Z^D."""
    Xp = layernorm(X, gamma, beta, eps, kind)
    return uniform_quant(Xp, np.asarray(s_ch, dtype=F64)[None, :], np.asarray(z_ch)[None, :], bits)


def reparam_fold(s_ch, z_ch, gamma, beta, W, b):
    """Channel-wise (s, z) -> layer-wise (s~, z~) with the variation folded away.

    s~ = E[s], z~ = E[z] (rounded to an integer so r2 is integral);
    r1 = s / s~, r2 = z - z~;
    beta~ = (beta + s.r2) / r1, gamma~ = gamma / r1          (Eq. raparm_1)
    W~[:, j] = r1 . W[:, j],  b~_j = b_j - (s.r2) W[:, j]     (Eq. raparm_2)

    W is stored [D_out, D] (row j = output channel j = the paper's column W[:, j]).
    Returns float64 arrays and Python scalars.
    """
    s = np.asarray(s_ch, dtype=F64)
    z = np.asarray(z_ch, dtype=np.int64)
    gamma = np.asarray(gamma, dtype=F64)
    beta = np.asarray(beta, dtype=F64)
    W = np.asarray(W, dtype=F64)
    b = np.asarray(b, dtype=F64)
    s_t = float(s.mean())
    z_t = int(np.rint(z.astype(F64).mean()))
    r1 = s / s_t
    r2 = (z - z_t).astype(F64)
    shift = s * r2
    beta_t = (beta + shift) / r1
    gamma_t = gamma / r1
    W_t = W * r1[None, :]
    b_t = b - W @ shift
    return dict(s_t=s_t, z_t=z_t, r1=r1, r2=r2, gamma_t=gamma_t, beta_t=beta_t, W_t=W_t, b_t=b_t)


def ln_quant(X, gamma_t, beta_t, s_t, z_t, bits, eps, kind=NORM_LAYERNORM):
    """Reparameterized tier: LayerNorm with the folded affine, then ONE scalar (s~, z~)."""
    Xt = layernorm(X, gamma_t, beta_t, eps, kind)
    return uniform_quant(Xt, F64(s_t), int(z_t), bits)


# --------------------------------------------------------------------------
# Weights: channel-wise (per output channel) uniform quantization
# (Section "Efficient quantizers", granularity paragraph; "Implementation details")
# --------------------------------------------------------------------------
def weight_quant(W, bits):
    """Per-output-channel min/max uniform quantization of W [D_out, K] (Eq. for s and z, per row of W).

    The zero-point of a weight row is itself a code: an integer in [0, 2^b - 1].  The formula z = round(-min / s) gives
    that exactly when the row's range contains 0; a row whose weights all share one sign has its range extended to 0
    (min(row, 0) .. max(row, 0)), so that z = 0 or 2^b - 1 and every weight stays inside the grid.  A row of zeros gets
    s = 1 (any positive scale represents it exactly).
    The scale is rounded to float32 (it is stored as float32) before the codes
    are taken, so codes and stored scale are consistent.
    Returns codes [D_out, K] (int64 in [0, 2^b-1]), s_w float32 [D_out], z_w int64 [D_out].
    """
    W = np.asarray(W, dtype=F64)
    lo = np.minimum(W.min(axis=1), 0.0)
    hi = np.maximum(W.max(axis=1), 0.0)
    s = ((hi - lo) / (2 ** bits - 1)).astype(np.float32)
    s = np.where(s > 0, s, np.float32(1.0)).astype(np.float32)
    s64 = s.astype(F64)
    z = np.rint(-lo / s64).astype(np.int64)
    codes = uniform_quant(W, s64[:, None], z[:, None], bits)
    return codes, s, z


# --------------------------------------------------------------------------
# Matmuls on codes (both operands quantized; Section "Transformer blocks", last paragraph)
# --------------------------------------------------------------------------
def int_matmul_nt(A, B):
    """Exact integer sum_k A[m,k] * B[n,k].  float64 BLAS is exact here: every partial
    sum is an integer below 2^53 (|a|,|b| <= 255, K <= 2^20)."""
    A = np.asarray(A)
    B = np.asarray(B)
    assert A.shape[-1] == B.shape[-1]
    assert A.shape[-1] * 255 * 255 < 2 ** 53
    acc = A.astype(F64) @ np.swapaxes(B.astype(F64), -1, -2)
    out = acc.astype(np.int64)
    assert np.all(np.abs(out) < 2 ** 31), "accumulator does not fit int32"
    return out


def qlinear_acc(qa, z_a, qw, z_w):
    """True integer accumulator sum_k (qa[m,k] - z_a) * (qw[n,k] - z_w[n])."""
    a = np.asarray(qa, dtype=np.int64) - int(z_a)
    w = np.asarray(qw, dtype=np.int64) - np.asarray(z_w, dtype=np.int64)[:, None]
    return int_matmul_nt(a, w)


def qlinear(qa, s_a, z_a, lin):
    """De-quantized Linear on codes: y = s_a * s_w[n] * acc[m, n] + bias[n]
    (the uniform de-quantizer applied to both operands of X W + b)."""
    acc = qlinear_acc(qa, z_a, lin["codes"], lin["z_w"])
    scale = F64(s_a) * np.asarray(lin["s_w"], dtype=F64)
    y = acc.astype(F64) * scale[None, :]
    if lin.get("bias") is not None:
        y = y + np.asarray(lin["bias"], dtype=F64)[None, :]
    return y


def gelu(x):
    """GELU, erf form: x/2 * (1 + erf(x / sqrt2))."""
    x = np.asarray(x, dtype=F64)
    return 0.5 * x * (1.0 + _erf(x / SQRT2))


def silu(x):
    x = np.asarray(x, dtype=F64)
    return x / (1.0 + np.exp(-x))


def softmax_rows(L):
    """Softmax over the last axis; -inf entries get exactly 0."""
    L = np.asarray(L, dtype=F64)
    m = L.max(axis=-1, keepdims=True)
    e = np.exp(L - m)
    return e / e.sum(axis=-1, keepdims=True)


def attention_logits(qq, z_q, s_q, qk, z_k, s_k, d_head, bias=None, causal=False):
    """Logits of one attention group: s_q s_k / sqrt(d_head) * sum_c (q - z_q)(k - z_k)  (+ bias),
    masked positions set to -inf.  Returns (logits float64, integer accumulators)."""
    acc = int_matmul_nt(np.asarray(qq, dtype=np.int64) - int(z_q),
                        np.asarray(qk, dtype=np.int64) - int(z_k))
    scale = F64(s_q) * F64(s_k) / math.sqrt(d_head)
    L = acc.astype(F64) * scale
    if bias is not None:
        L = L + np.asarray(bias, dtype=F64)
    if causal:
        n_q, n_k = L.shape
        L = np.where(np.arange(n_k)[None, :] > np.arange(n_q)[:, None], -np.inf, L)
    return L, acc


def softmax_log_quant(L, s_log, bits):
    """Softmax, then the log-sqrt2 quantizer in its base-2 form (Eq. (3.3-1), second line)."""
    return logsqrt2_quant_base2(softmax_rows(L), s_log, bits)


def attn_pv(codes, qv, s_log, s_v, z_v, causal=False, bits=None, zero_at_max=False):
    """P.V with shift-form de-quantized probabilities:
    out[i, c] = sum_j s~(code_ij) 2^floor(-code_ij / 2) * s_v (v[j, c] - z_v); masked j excluded."""
    P = logsqrt2_dequant_shift(codes, s_log, bits, zero_at_max)
    if causal:
        n_q, n_k = P.shape
        P = np.where(np.arange(n_k)[None, :] > np.arange(n_q)[:, None], 0.0, P)
    V = uniform_dequant(qv, s_v, z_v)
    return P @ V


def attn_pv_sqrt2(codes, qv, s_log, s_v, z_v, causal=False, bits=None, zero_at_max=False):
    """Definition tier of the same product: probabilities de-quantized as s * sqrt2^(-q)."""
    P = logsqrt2_dequant(codes, s_log, bits, zero_at_max)
    if causal:
        n_q, n_k = P.shape
        P = np.where(np.arange(n_k)[None, :] > np.arange(n_q)[:, None], 0.0, P)
    return P @ uniform_dequant(qv, s_v, z_v)


# --------------------------------------------------------------------------
# The block (Eqs. for X-bar and Y; attention Eq.)
# --------------------------------------------------------------------------
def block_forward(P, x, keep=False):
    """Quantized, reparameterized block:
        X-bar = MSA(LayerNorm(X)) + X,  Y = MLP(LayerNorm(X-bar)) + X-bar,
    every matmul operand quantized.  `P` is the dict produced by calibrate_block
    (or the same fields from anywhere else).  x is [batch*seq, D].
    Returns y (float64) and, with keep=True, every intermediate tensor."""
    c = P["cfg"]
    D, H, seq, batch = c["D"], c["H"], c["seq"], c["batch"]
    dh = D // H
    ba, bp = c["bits_a"], c["bits_p"]
    causal = c["mask"] == MASK_CAUSAL
    zero_max = bool(c.get("log_zero_at_max_code", False))
    X = np.asarray(x, dtype=F64)
    T = X.shape[0]
    assert T == batch * seq
    t = {}

    ln1 = P["ln1"]
    a1 = ln_quant(X, ln1["gamma_t"], ln1["beta_t"], ln1["s"], ln1["z"], ba, c["eps"], c["norm"])
    qkv = qlinear(a1, ln1["s"], ln1["z"], P["qkv"])
    qq = uniform_quant(qkv[:, 0:D], P["s_q"], P["z_q"], ba)
    qk = uniform_quant(qkv[:, D:2 * D], P["s_k"], P["z_k"], ba)
    qv = uniform_quant(qkv[:, 2 * D:3 * D], P["s_v"], P["z_v"], ba)

    attn = np.empty((T, D), dtype=F64)
    codes_all = np.empty((batch, H, seq, seq), dtype=np.uint8) if keep else None
    acc_all = np.empty((batch, H, seq, seq), dtype=np.int32) if keep else None
    for b in range(batch):
        r = slice(b * seq, (b + 1) * seq)
        for h in range(H):
            cs = slice(h * dh, (h + 1) * dh)
            bias = None if P.get("rel_bias") is None else P["rel_bias"][h]
            L, acc = attention_logits(qq[r, cs], P["z_q"], P["s_q"], qk[r, cs], P["z_k"], P["s_k"],
                                      dh, bias, causal)
            codes = softmax_log_quant(L, P["s_log"], bp)
            attn[r, cs] = attn_pv(codes, qv[r, cs], P["s_log"], P["s_v"], P["z_v"], causal, bp, zero_max)
            if keep:
                codes_all[b, h] = codes
                acc_all[b, h] = acc
    qo = uniform_quant(attn, P["s_o"], P["z_o"], ba)
    xbar = qlinear(qo, P["s_o"], P["z_o"], P["proj"]) + X

    ln2 = P["ln2"]
    a2 = ln_quant(xbar, ln2["gamma_t"], ln2["beta_t"], ln2["s"], ln2["z"], ba, c["eps"], c["norm"])
    h1 = qlinear(a2, ln2["s"], ln2["z"], P["fc1"])
    hid = mlp_activation(h1, c["act"], c["Dm"])
    qh = uniform_quant(hid, P["s_h"], P["z_h"], ba)
    y = qlinear(qh, P["s_h"], P["z_h"], P["fc2"]) + xbar
    if keep:
        t.update(a1=a1, qkv=qkv, qq=qq, qk=qk, qv=qv, attn=attn, qo=qo, xbar=xbar, a2=a2,
                 h1=h1, hid=hid, qh=qh, codes=codes_all, acc=acc_all)
        return y, t
    return y


def mlp_activation(h1, act, Dm):
    """GELU(h), or SiLU(gate) * up for the gated MLP (gate = first Dm columns, up = next Dm)."""
    if act == ACT_GELU:
        return gelu(h1)
    return silu(h1[:, :Dm]) * h1[:, Dm:2 * Dm]


# --------------------------------------------------------------------------
# Calibration of one block on one batch, in the order of Algorithm 1
# (activation quantizer -> reparameterization -> weight quantization, layer by layer,
#  each layer seeing the already-quantized layers before it).
# Weight quantization is round-to-nearest min/max (GPTQ is outside this build);
# non-LayerNorm activations take min/max bounds.
# --------------------------------------------------------------------------
def _f32(v):
    return np.asarray(v, dtype=F64).astype(np.float32)


def _lin(W, b, bits, A_int=None):
    """Weight quantization of one Linear: round-to-nearest on the per-channel min/max grid, or -- when the layer's
    integer-valued input codes A_int [T, K] are given -- GPTQ against them (Algorithm 1, last step of a layer)."""
    if A_int is None:
        codes, s_w, z_w = weight_quant(_f32(W), bits)
    else:
        from . import gptq_oracle
        codes, s_w, z_w = gptq_oracle.gptq(_f32(W), A_int, bits)
    return dict(codes=codes, s_w=s_w, z_w=z_w, bias=_f32(b))


def _tensor_qparams(v, bits):
    """Layer-wise (s, z) from the tensor's min/max; the scale is stored float32 and z follows it."""
    lo, hi = F64(v.min()), F64(v.max())
    s = np.float32((hi - lo) / (2 ** bits - 1))
    z = int(np.rint(-lo / F64(s)))
    return s, z


def _fold_ln(Xin, gamma, beta, W, b, clip_up, clip_lo, c, learn_clip=None):
    Xp = layernorm(Xin, gamma, beta, c["eps"], c["norm"])
    if learn_clip is not None:
        # Algorithm 1, "Per-channel dual clipping": the factors are learnt on this layer's X'; they are kept as float32
        from . import dual_clip_oracle
        r = dual_clip_oracle.learn(Xp, c["bits_a"], **learn_clip)
        clip_up, clip_lo = r["clip_up"].astype(np.float32), r["clip_lo"].astype(np.float32)
    lo, up = channel_bounds(Xp, clip_up, clip_lo)
    s_ch, _ = qparams_from_bounds(lo, up, c["bits_a"])
    s_ch = s_ch.astype(np.float32)                       # channel scales are stored float32
    z_ch = np.rint(-lo / s_ch.astype(F64)).astype(np.int64)
    f = reparam_fold(s_ch, z_ch, gamma, beta, W, b)
    ln = dict(gamma_t=_f32(f["gamma_t"]), beta_t=_f32(f["beta_t"]), s=np.float32(f["s_t"]), z=int(f["z_t"]),
              s_ch=s_ch, z_ch=z_ch)
    return ln, _f32(f["W_t"]), _f32(f["b_t"])


def calibrate_block(raw, cfg, learn_clip=None, gptq=False):
    """raw: dict of float32 arrays (x, ln1_gamma, ln1_beta, w_qkv, b_qkv, w_proj, b_proj, ln2_*, w_fc1,
    b_fc1, w_fc2, b_fc2, rel_bias, ln*_clip_up/lo); cfg: dict (batch, seq, D, H, Dm, bits_w, bits_a,
    bits_p, norm, act, mask, eps; optional log_zero_at_max_code).  Returns the parameter dict block_forward consumes.
    learn_clip: None (use the given clip factors) or dict(iters, lr, alpha0) -- learn them per LayerNorm (Algorithm 1);
    gptq: quantize every Linear with GPTQ against the codes it is fed, instead of round-to-nearest."""
    c = dict(cfg)
    D, H, seq, batch = c["D"], c["H"], c["seq"], c["batch"]
    dh = D // H
    ba, bw, bp = c["bits_a"], c["bits_w"], c["bits_p"]
    causal = c["mask"] == MASK_CAUSAL
    zero_max = bool(c.get("log_zero_at_max_code", False))
    X = np.asarray(raw["x"], dtype=F64)
    P = dict(cfg=c, s_log=np.float32(1.0), rel_bias=raw.get("rel_bias"))

    ln1, Wt, bt = _fold_ln(X, raw["ln1_gamma"], raw["ln1_beta"], raw["w_qkv"], raw["b_qkv"],
                           raw.get("ln1_clip_up"), raw.get("ln1_clip_lo"), c, learn_clip)
    P["ln1"] = ln1
    a1 = ln_quant(X, ln1["gamma_t"], ln1["beta_t"], ln1["s"], ln1["z"], ba, c["eps"], c["norm"])
    P["qkv"] = _lin(Wt, bt, bw, a1 - ln1["z"] if gptq else None)
    qkv = qlinear(a1, ln1["s"], ln1["z"], P["qkv"])
    for i, nm in enumerate("qkv"):
        P["s_" + nm], P["z_" + nm] = _tensor_qparams(qkv[:, i * D:(i + 1) * D], ba)
    qq = uniform_quant(qkv[:, 0:D], P["s_q"], P["z_q"], ba)
    qk = uniform_quant(qkv[:, D:2 * D], P["s_k"], P["z_k"], ba)
    qv = uniform_quant(qkv[:, 2 * D:3 * D], P["s_v"], P["z_v"], ba)
    attn = np.empty_like(X)
    for b in range(batch):
        r = slice(b * seq, (b + 1) * seq)
        for h in range(H):
            cs = slice(h * dh, (h + 1) * dh)
            bias = None if P["rel_bias"] is None else P["rel_bias"][h]
            L, _ = attention_logits(qq[r, cs], P["z_q"], P["s_q"], qk[r, cs], P["z_k"], P["s_k"], dh, bias, causal)
            codes = softmax_log_quant(L, P["s_log"], bp)
            attn[r, cs] = attn_pv(codes, qv[r, cs], P["s_log"], P["s_v"], P["z_v"], causal, bp, zero_max)
    P["s_o"], P["z_o"] = _tensor_qparams(attn, ba)
    qo = uniform_quant(attn, P["s_o"], P["z_o"], ba)
    P["proj"] = _lin(raw["w_proj"], raw["b_proj"], bw, qo - P["z_o"] if gptq else None)
    xbar = qlinear(qo, P["s_o"], P["z_o"], P["proj"]) + X

    ln2, Wt, bt = _fold_ln(xbar, raw["ln2_gamma"], raw["ln2_beta"], raw["w_fc1"], raw["b_fc1"],
                           raw.get("ln2_clip_up"), raw.get("ln2_clip_lo"), c, learn_clip)
    P["ln2"] = ln2
    a2 = ln_quant(xbar, ln2["gamma_t"], ln2["beta_t"], ln2["s"], ln2["z"], ba, c["eps"], c["norm"])
    P["fc1"] = _lin(Wt, bt, bw, a2 - ln2["z"] if gptq else None)
    hid = mlp_activation(qlinear(a2, ln2["s"], ln2["z"], P["fc1"]), c["act"], c["Dm"])
    P["s_h"], P["z_h"] = _tensor_qparams(hid, ba)
    qh = uniform_quant(hid, P["s_h"], P["z_h"], ba)
    P["fc2"] = _lin(raw["w_fc2"], raw["b_fc2"], bw, qh - P["z_h"] if gptq else None)
    return P


# --------------------------------------------------------------------------
# Definition-tier block pieces used by the pins
# --------------------------------------------------------------------------
def ln_linear_channelwise(X, gamma, beta, s_ch, z_ch, W, b, bits, eps, kind=NORM_LAYERNORM):
    """LayerNorm -> channel-wise quant -> de-quant -> X^' W + b with the ORIGINAL W, b."""
    q = ln_quant_channelwise(X, gamma, beta, s_ch, z_ch, bits, eps, kind)
    Xhat = uniform_dequant(q, np.asarray(s_ch, dtype=F64)[None, :], np.asarray(z_ch)[None, :])
    return q, Xhat @ np.asarray(W, dtype=F64).T + np.asarray(b, dtype=F64)[None, :]


def ln_linear_layerwise(X, fold, bits, eps, kind=NORM_LAYERNORM):
    """LayerNorm with folded affine -> layer-wise quant -> de-quant -> X~^' W~ + b~."""
    q = ln_quant(X, fold["gamma_t"], fold["beta_t"], fold["s_t"], fold["z_t"], bits, eps, kind)
    Xhat = uniform_dequant(q, fold["s_t"], fold["z_t"])
    return q, Xhat @ fold["W_t"].T + fold["b_t"][None, :]

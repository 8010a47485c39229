"""CPU oracle for GPTQ weight reconstruction on the folded weights -- TEST INFRASTRUCTURE ONLY.

Algorithm 1 of arXiv 2402.05628 ends every layer with "perform GPTQ to quantize the layer's weights", applied to the
weights the scale reparameterization has just updated (Section "Sequential Quantization Pipeline").  GPTQ itself is the
published method of Frantar et al. (2022): quantize the columns of W one after the other and, after each one, move the
not-yet-quantized columns so that the layer's output error  ||W X^T - W^ X^T||^2  over the calibration inputs stays
as small as the second-order model allows.

This file states that procedure in its plain elimination form, float64 numpy, no Cholesky factor and no blocking:

    H = X^T X  (+ damping),   Hinv = H^-1
    for j = 0 .. K-1:
        q_j   = quantize(w_j)                        (every output channel with its own fixed grid)
        delta = (w_j - dequant(q_j)) / Hinv[j, j]
        W[:, j+1:] -= delta (x) Hinv[j, j+1:]        (optimal compensation given that column j is now fixed)
        Hinv[j+1:, j+1:] -= Hinv[j+1:, j] (x) Hinv[j, j+1:] / Hinv[j, j]      (inverse Hessian of the remaining columns)

The HIP library computes the same thing from a Cholesky factor of the inverse Hessian, in column blocks; the two share
no code.  Only tests/, smoke() and the cpu_baseline leg of the benchmark may import this module.

Readings (this paper only names the method; the conventions below follow the published description of GPTQ):
  * calibration inputs are the layer's inputs as the quantized model sees them, i.e. the de-quantized activation codes
    s_a (q - z_a); the Hessian's scale cancels, so H is taken as the exact integer Gram matrix of (q - z_a);
  * damping: lambda = percdamp * mean(diag H) added to the diagonal, percdamp = 0.01;
  * a column whose inputs are all zero (H_jj = 0) gets H_jj = 1 and its weights are set to 0 before anything else;
  * natural column order; per-output-channel min/max grid taken from the weights BEFORE the sweep (after the zeroing
    above), scale stored as float32, round-half-to-even -- the same grid as the round-to-nearest weight quantizer.
Parity unpinned by the paper (it prints no GPTQ values): the pins are special cases with closed forms, the optimality
condition of one compensation step solved independently, and the Cholesky formulation evaluated with library routines
(tests/test_gptq_pins.py).
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


def gram_matrix(A_int):
    """H = A^T A for integer-valued activations (q - z_a).  Taken in float64, where it is exact: every partial sum is an
    integer below 2^53 (|a| <= 255, T < 10^11), whatever the order of the additions."""
    A = np.asarray(A_int, dtype=F64)
    assert np.array_equal(A, np.rint(A)) and np.abs(A).max(initial=0) <= 255
    return A.T @ A


def damped_hessian(H, W, percdamp=0.01):
    """Dead columns and damping.  Returns (H', W') -- copies."""
    H = np.array(H, dtype=F64)
    W = np.array(W, dtype=F64)
    dead = np.diag(H) == 0
    H[dead, dead] = 1.0
    W[:, dead] = 0.0
    H[np.diag_indices_from(H)] += percdamp * np.mean(np.diag(H))
    return H, W


def row_grid(W, bits):
    """Per-output-channel min/max grid (Eq. for s and z per row of W); the scale is a float32 number.  As in the
    round-to-nearest weight quantizer the row's range is taken to contain 0, so that z is a code in [0, 2^b - 1]."""
    lo, hi = np.minimum(W.min(axis=1), 0.0), np.maximum(W.max(axis=1), 0.0)
    s = ((hi - lo) / (2 ** bits - 1)).astype(np.float32).astype(F64)
    s = np.where(s > 0, s, 1.0)
    z = np.rint(-lo / s)
    return s, z


def gptq(W, A_int, bits, percdamp=0.01):
    """GPTQ of W [N, K] against integer-valued calibration inputs A_int [T, K].

    Returns codes [N, K] (int64 in [0, 2^b - 1]), s_w float32 [N], z_w int64 [N].
    """
    H, Wc = damped_hessian(gram_matrix(A_int), W, percdamp)
    N, K = Wc.shape
    qmax = 2 ** bits - 1
    s, z = row_grid(Wc, bits)
    Hinv = np.linalg.inv(H)
    codes = np.zeros((N, K), dtype=np.int64)
    for j in range(K):
        q = np.clip(np.rint(Wc[:, j] / s) + z, 0, qmax)
        codes[:, j] = q.astype(np.int64)
        d = Hinv[j, j]
        delta = (Wc[:, j] - s * (q - z)) / d
        Wc[:, j + 1:] -= np.outer(delta, Hinv[j, j + 1:])
        Hinv[j + 1:, j + 1:] -= np.outer(Hinv[j + 1:, j], Hinv[j, j + 1:]) / d
    return codes, s.astype(np.float32), z.astype(np.int64)


def output_error(W, codes, s, z, A_int):
    """|| (W - W^) A^T ||_F^2 over the calibration inputs."""
    Wq = np.asarray(s, dtype=F64)[:, None] * (codes.astype(F64) - np.asarray(z, dtype=F64)[:, None])
    R = (np.asarray(W, dtype=F64) - Wq) @ np.asarray(A_int, dtype=F64).T
    return float((R * R).sum())

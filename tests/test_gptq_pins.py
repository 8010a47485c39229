"""Pins for the GPTQ oracle (Algorithm 1, weight-quantization step): special cases that reduce to round-to-nearest, the
conditional least-squares problem every column's value solves (re-solved from scratch with numpy), the Cholesky
formulation of the same sweep evaluated with scipy, and invariances.  CPU only."""
import numpy as np
import pytest
import scipy.linalg

from oracle import gptq_oracle as gq
from oracle import repquant_oracle as orc


def _case(N, K, T, bits_a=4, seed=0, corr=0.7):
    g = np.random.default_rng(seed)
    W = (g.standard_normal((N, K)) * 0.05).astype(np.float32)
    base = g.standard_normal((T, 1))
    X = corr * base + (1 - corr) * g.standard_normal((T, K))          # correlated channels: compensation matters
    qmax = 2 ** bits_a - 1
    A = np.clip(np.rint(X * 2.5) + qmax // 2, 0, qmax).astype(np.int64) - qmax // 2
    return W, A


def test_uncorrelated_inputs_reduce_to_round_to_nearest():
    """Diagonal Hessian: the inverse has no off-diagonal entries, nothing is compensated."""
    g = np.random.default_rng(1)
    W = (g.standard_normal((7, 16)) * 0.1).astype(np.float32)
    A = np.diag(g.integers(1, 8, size=16)).astype(np.int64)           # each token excites one channel
    codes, s, z = gq.gptq(W, A, 4)
    want, s_w, z_w = orc.weight_quant(W, 4)
    assert np.array_equal(codes, want) and np.array_equal(s, s_w) and np.array_equal(z, z_w)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_every_column_is_the_conditional_least_squares_refit(seed):
    """With e = W - W^ and the damped Hessian H, the error is e H e^T per row.  Once columns P = {0..j-1} are fixed, the
    best continuous values of the remaining columns F are W_F + E_P H_PF H_FF^-1; GPTQ quantizes the first of them."""
    W, A = _case(5, 8, 64, seed=seed)
    bits = 3
    codes, s, z = gq.gptq(W, A, bits)
    H, Wd = gq.damped_hessian(gq.gram_matrix(A), W)
    s64, z64 = s.astype(np.float64), z.astype(np.float64)
    Wq = s64[:, None] * (codes - z64[:, None])
    for j in range(8):
        E_P = Wd[:, :j] - Wq[:, :j]
        refit = Wd[:, j:] + (E_P @ H[:j, j:]) @ np.linalg.inv(H[j:, j:]) if j else Wd[:, j:]
        want = np.clip(np.rint(refit[:, 0] / s64) + z64, 0, 2 ** bits - 1)
        assert np.array_equal(codes[:, j], want.astype(np.int64)), j


def test_cholesky_formulation_gives_the_same_codes():
    """The published fast form: U = upper Cholesky factor of H^-1; err_j = (w_j - dq_j) / U_jj; W[:, j+1:] -= err_j U[j, j+1:]."""
    W, A = _case(12, 48, 300, seed=5)
    bits = 4
    codes, s, z = gq.gptq(W, A, bits)
    H, Wc = gq.damped_hessian(gq.gram_matrix(A), W)
    U = scipy.linalg.cholesky(scipy.linalg.inv(H), lower=False)
    s64, z64 = s.astype(np.float64), z.astype(np.float64)
    got = np.zeros_like(codes)
    for j in range(48):
        q = np.clip(np.rint(Wc[:, j] / s64) + z64, 0, 15)
        got[:, j] = q
        err = (Wc[:, j] - s64 * (q - z64)) / U[j, j]
        Wc[:, j + 1:] -= np.outer(err, U[j, j + 1:])
    assert np.array_equal(got, codes)


def test_lower_output_error_than_round_to_nearest_on_correlated_inputs():
    W, A = _case(32, 64, 512, seed=3)
    codes, s, z = gq.gptq(W, A, 3)
    rtn, s_r, z_r = orc.weight_quant(W, 3)
    assert np.array_equal(s, s_r) and np.array_equal(z, z_r)             # same grid, different codes
    assert not np.array_equal(codes, rtn)
    assert gq.output_error(W, codes, s, z, A) < 0.7 * gq.output_error(W, rtn, s_r, z_r, A)


def test_dead_input_channel():
    W, A = _case(6, 16, 100, seed=4)
    A[:, 5] = 0
    codes, s, z = gq.gptq(W, A, 4)
    assert np.all(codes[:, 5] == np.clip(z, 0, 15))                      # weight forced to 0 -> code z
    W2 = W.copy()
    W2[:, 5] = 7.0                                                       # whatever stood there is irrelevant
    codes2, s2, z2 = gq.gptq(W2, A, 4)
    assert np.array_equal(codes, codes2) and np.array_equal(s, s2)


def test_input_scale_and_output_channel_independence():
    W, A = _case(10, 24, 200, seed=6)
    codes, s, z = gq.gptq(W, A, 4)
    codes3, _, _ = gq.gptq(W, 3 * A, 4)                                  # the Hessian's scale cancels (damping is relative)
    assert np.array_equal(codes, codes3)
    sub, s_sub, _ = gq.gptq(W[[7, 1, 4]], A, 4)
    assert np.array_equal(sub, codes[[7, 1, 4]]) and np.array_equal(s_sub, s[[7, 1, 4]])

"""Pins for the random-projection scheme of the oracle (Section 3.2, last
paragraph; Appendix "Random projections for RAD"): P = R R^T / k with R a
d x k matrix of independent signs.  What fixes it: diag(P) = 1 exactly,
E[P] = I, the closed-form variance of P v, sign balance and independence, and
that the stored object is k numbers per row."""
import numpy as np
import pytest

from oracle import rad_oracle as R


def test_sign_bits_by_big_integers():
    d, p = 37, 0.3
    k = R.fixed_k(p, d)
    Rm = R.rademacher_matrix(p, 77, 5, 2, d)
    assert Rm.shape == (d, k) and set(np.unique(Rm)) == {-1.0, 1.0}
    words = R.element_keys(77, 5, 2, 0, (d * k + 31) // 32)
    for j in range(d):
        for s in range(k):
            f = j * k + s
            bit = (int(words[f // 32]) >> (f % 32)) & 1
            assert Rm[j, s] == (1.0 if bit == 0 else -1.0)


def test_signs_are_balanced_and_independent():
    d, p = 2048, 0.1
    Rm = R.rademacher_matrix(p, 1, 0, 0, d)
    k = Rm.shape[1]
    n = d * k
    assert abs(Rm.mean()) < 5 / np.sqrt(n)
    # columns are nearly orthogonal: entries of R^T R / d off the diagonal are N(0, 1/d)
    G = Rm.T @ Rm / d
    off = G[~np.eye(k, dtype=bool)]
    assert np.all(np.diag(G) == 1.0)
    assert abs(off.std() * np.sqrt(d) - 1) < 0.05 and np.abs(off).max() < 6 / np.sqrt(d)
    # a different stream or step gives an unrelated matrix
    R2 = R.rademacher_matrix(p, 1, 1, 0, d)
    assert abs((Rm * R2).mean()) < 5 / np.sqrt(n)


def test_P_has_unit_diagonal_and_mean_identity():
    d, p, S = 24, 0.25, 3000
    k = R.fixed_k(p, d)
    acc = np.zeros((d, d))
    for s in range(S):
        Rm = R.rademacher_matrix(p, s, 0, 0, d)
        P = Rm @ Rm.T / k
        assert np.all(np.diag(P) == 1.0)
        acc += P
    mean = acc / S
    off = mean[~np.eye(d, dtype=bool)]
    assert np.abs(off).max() < 5 / np.sqrt(k * S)          # Var P_ij = 1/k for i != j
    # P is a rank-k matrix, not the identity, even at the full fraction
    Rfull = R.rademacher_matrix(1.0, 0, 0, 0, d)
    assert not np.allclose(Rfull @ Rfull.T / d, np.eye(d))


def test_store_is_k_numbers_per_row_and_xt_is_xP():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((7, 120)).astype(np.float32)
    rp, col, val, xt = R.sample_pack(x, R.PROJECT_SHARED, 0.1, 9, 1, 0)
    k = R.fixed_k(0.1, 120)
    assert np.array_equal(rp, np.arange(8) * k) and len(val) == 7 * k
    Rm = R.rademacher_matrix(0.1, 9, 1, 0, 120)
    want = x.astype(np.float64) @ (Rm @ Rm.T) / k
    assert np.abs(xt - want).max() < 1e-5 * np.abs(want).max()     # z is rounded to fp32 once
    z16 = R.sample_pack(x, R.PROJECT_SHARED, 0.1, 9, 1, 0, R.BF16)[2]
    assert np.array_equal(z16, R.round_bf16(z16)) and np.abs(z16 - val).max() < 2 ** -7 * np.abs(val).max()


def test_unbiased_and_variance_closed_form():
    """(P v)_j = v_j + (1/k) sum_s sum_{i != j} R_js R_is v_i, so Var (P v)_j = (|v|^2 - v_j^2) / k."""
    rng = np.random.default_rng(17)
    B, D, N, p, S = 9, 32, 4, 0.25, 6000
    x = rng.standard_normal((B, D)).astype(np.float32)
    dy = rng.standard_normal((B, N)).astype(np.float32)
    bits = rng.random((B, N)) > 0.3
    exact = x.astype(np.float64).T @ (dy.astype(np.float64) * bits)
    acc = np.zeros_like(exact)
    acc2 = np.zeros_like(exact)
    for s in range(S):
        e = R.backward_dW(R.sample_pack(x, R.PROJECT_SHARED, p, s, 1, 0)[3], dy, bits)
        acc += e
        acc2 += e * e
    mean = acc / S
    var = acc2 / S - mean**2
    k = R.fixed_k(p, D)
    var_cf = ((exact**2).sum(axis=0, keepdims=True) - exact**2) / k
    err = np.linalg.norm(mean - exact)
    assert 0 < err < 4 * np.sqrt(var_cf.sum() / S)
    assert abs(var.sum() / var_cf.sum() - 1) < 0.08
    assert np.abs(var / var_cf - 1).max() < 0.35               # element by element as well


def test_train_step_keeps_the_exact_chain():
    rng = np.random.default_rng(4)
    dims = [20, 16, 12, 5]
    x = rng.standard_normal((10, 20)).astype(np.float32)
    Ws = [(rng.standard_normal((dims[i], dims[i + 1])) / np.sqrt(dims[i])).astype(np.float32) for i in range(3)]
    bs = [np.zeros(dims[i + 1], np.float32) for i in range(3)]
    labels = rng.integers(0, 5, 10).astype(np.int32)
    ref = R.mlp_train_step(x, labels, Ws, bs, R.EXACT, 1.0, seed=0)
    out = R.mlp_train_step(x, labels, Ws, bs, R.PROJECT_SHARED, 0.3, seed=2)
    assert out["loss"] == ref["loss"]
    for l in range(3):
        assert np.array_equal(out["dy"][l], ref["dy"][l])
        assert not np.array_equal(out["dW"][l], ref["dW"][l])

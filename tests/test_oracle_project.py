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


# ------------------------------------------------------------------ a matrix of its own for every example
def test_per_example_sign_bits_by_big_integers():
    """Row (b, j) owns whole Philox calls: 4 ceil(k/128) keys from flat index (b d + j) 4 ceil(k/128) on."""
    for d, p in ((21, 0.4), (400, 0.4)):            # k = 9 (one call per row), k = 160 (two)
        k = R.fixed_k(p, d)
        wpr = 4 * ((k + 127) // 128)
        for b in (0, 3):
            Rb = R.rademacher_matrix_of_example(p, 5, 2, 1, b, d)
            assert Rb.shape == (d, k) and set(np.unique(Rb)) == {-1.0, 1.0}
            for j in (0, 1, d - 1):
                words = R.element_keys(5, 2, 1, (b * d + j) * wpr, wpr)
                for s in range(k):
                    bit = (int(words[s // 32]) >> (s % 32)) & 1
                    assert Rb[j, s] == (1.0 if bit == 0 else -1.0)


def test_per_example_matrices_are_unrelated():
    d, p = 512, 0.25
    R0 = R.rademacher_matrix_of_example(p, 1, 0, 0, 0, d)
    R1 = R.rademacher_matrix_of_example(p, 1, 0, 0, 1, d)
    n = R0.size
    assert abs(R0.mean()) < 5 / np.sqrt(n) and abs((R0 * R1).mean()) < 5 / np.sqrt(n)
    assert abs((R0[1:] * R0[:-1]).mean()) < 5 / np.sqrt(n)        # neighbouring rows
    assert abs((R0[:, 1:] * R0[:, :-1]).mean()) < 5 / np.sqrt(n)  # neighbouring columns


def test_per_example_store_is_x_times_its_own_P():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((5, 150)).astype(np.float32)
    rp, col, val, xt = R.sample_pack(x, R.PROJECT_PER_EXAMPLE, 0.2, 4, 1, 0)
    k = R.fixed_k(0.2, 150)
    assert np.array_equal(rp, np.arange(6) * k) and len(val) == 5 * k
    for b in range(5):
        Rb = R.rademacher_matrix_of_example(0.2, 4, 1, 0, b, 150)
        want = x[b].astype(np.float64) @ (Rb @ Rb.T) / k
        assert np.abs(xt[b] - want).max() < 1e-5 * np.abs(want).max()


def test_per_example_unbiased_and_variance_closed_form():
    """The examples' matrices are independent, so the variances of their contributions add:
    Var dW~[j, n] = sum_b g[b, n]^2 (|x_b|^2 - x[b, j]^2) / k."""
    rng = np.random.default_rng(18)
    B, D, N, p, S = 6, 32, 3, 0.25, 6000
    x = rng.standard_normal((B, D)).astype(np.float32)
    dy = rng.standard_normal((B, N)).astype(np.float32)
    bits = rng.random((B, N)) > 0.3
    g = dy.astype(np.float64) * bits
    exact = x.astype(np.float64).T @ g
    acc = np.zeros_like(exact); acc2 = np.zeros_like(exact)
    for s in range(S):
        e = R.backward_dW(R.sample_pack(x, R.PROJECT_PER_EXAMPLE, p, s, 1, 0)[3], dy, bits)
        acc += e; acc2 += e * e
    mean = acc / S
    var = acc2 / S - mean**2
    k = R.fixed_k(p, D)
    x64 = x.astype(np.float64)
    var_cf = (((x64**2).sum(axis=1, keepdims=True) - x64**2).T @ g**2) / k
    err = np.linalg.norm(mean - exact)
    assert 0 < err < 4 * np.sqrt(var_cf.sum() / S)
    assert abs(var.sum() / var_cf.sum() - 1) < 0.08
    assert np.abs(var / var_cf - 1).max() < 0.35
    # and it differs from the shared-matrix variance, whose cross terms between examples do not vanish
    var_shared = ((exact**2).sum(axis=0, keepdims=True) - exact**2) / k
    assert abs(var_shared.sum() / var_cf.sum() - 1) > 0.1

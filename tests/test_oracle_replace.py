"""Pins for the with-replacement sampling schemes of the oracle: the matrix
P = (d/k) sum_s e_{i_s} e_{i_s}^T of Section 3.2 with k uniform independent
draws.  What fixes it: the draws of a row number k, their counts are
Binomial(k, 1/d), E[P] = I, the variance of the estimate has a closed form, and
(Appendix A, fraction-sweep caption) the full fraction does not give back the
baseline because indices repeat."""
import numpy as np
import pytest

from oracle import rad_oracle as R


def test_index_map_by_big_integers():
    """i = floor(key d / 2^32), recomputed with Python integers; every index owns floor or ceil of 2^32/d keys."""
    for d, k_rows in ((7, 3), (300, 2), (4096, 1), (65535, 1)):
        p = 0.5
        k = R.fixed_k(p, d)
        idx = R.replace_draws(R.REPLACE_PER_EXAMPLE, p, 99, 4, 2, k_rows, d)
        keys = R.element_keys(99, 4, 2, 0, k_rows * k).reshape(k_rows, k)
        for b in range(k_rows):
            for s in range(0, k, max(1, k // 50)):
                assert idx[b, s] == (int(keys[b, s]) * d) // (1 << 32)
        assert idx.min() >= 0 and idx.max() < d
    # the map itself at its edges
    for d in (1, 3, 1000):
        for key, want in ((0, 0), ((1 << 32) - 1, d - 1), ((1 << 32) // d, 1 if d > 1 else 0)):
            got = (np.uint64(key) * np.uint64(d)) >> np.uint64(32)
            assert int(got) == (key * d) // (1 << 32) and (d == 1 or key != (1 << 32) // d or int(got) in (0, want))


def test_draws_number_k_and_shared_rows_agree():
    for scheme in (R.REPLACE_SHARED, R.REPLACE_PER_EXAMPLE):
        m = R.multiplicity(scheme, 0.1, 5, 0, 0, 9, 300)
        assert np.all(m.sum(axis=1) == R.fixed_k(0.1, 300))
        if scheme == R.REPLACE_SHARED:
            assert np.all(m == m[0])
        else:
            assert not np.all(m == m[0])
    # shared: the draws do not depend on the number of rows; per example: row b does not depend on other rows
    a = R.replace_draws(R.REPLACE_PER_EXAMPLE, 0.2, 1, 2, 3, 4, 50)
    b = R.replace_draws(R.REPLACE_PER_EXAMPLE, 0.2, 1, 2, 3, 9, 50)
    assert np.array_equal(a, b[:4])


def test_counts_are_binomial():
    d, p, rows = 200, 0.25, 4000
    k = R.fixed_k(p, d)
    m = R.multiplicity(R.REPLACE_PER_EXAMPLE, p, 2024, 1, 0, rows, d)
    n = rows * d
    q = 1.0 / d
    mean, var = k * q, k * q * (1 - q)
    assert abs(m.mean() - mean) < 5 * np.sqrt(var / n)
    # fourth central moment of a binomial bounds the error of the variance estimate
    mu4 = k * q * (1 - q) * (1 + 3 * (k - 2) * q * (1 - q))
    assert abs(m.var() - var) < 5 * np.sqrt((mu4 - var**2) / n) + 5 * var / n
    # number of distinct coordinates of a row
    distinct = (m > 0).sum(axis=1)
    want = d * (1 - (1 - q) ** k)
    assert abs(distinct.mean() - want) < 5 * distinct.std() / np.sqrt(rows)
    assert distinct.max() <= k
    # every coordinate is drawn equally often: chi-square over all rows
    col = m.sum(axis=0)
    chi2 = ((col - rows * k / d) ** 2 / (rows * k / d)).sum()
    assert abs(chi2 - (d - 1)) < 6 * np.sqrt(2 * (d - 1))


def test_full_fraction_is_not_the_baseline():
    """Appendix A (fraction sweep): with replacement even the full fraction keeps repeating indices."""
    rng = np.random.default_rng(0)
    x = rng.standard_normal((6, 64)).astype(np.float32) + 2
    xt_r = R.sample_pack(x, R.REPLACE_PER_EXAMPLE, 1.0, 3, 0, 0)[3]
    xt_w = R.sample_pack(x, R.FIXEDK_PER_EXAMPLE, 1.0, 3, 0, 0)[3]
    assert np.array_equal(xt_w, x)
    assert not np.array_equal(xt_r, x)
    m = R.multiplicity(R.REPLACE_PER_EXAMPLE, 1.0, 3, 0, 0, 6, 64)
    assert np.all((m == 0).sum(axis=1) > 0) and np.all(m.sum(axis=1) == 64)
    # weights are the counts: scale is d/k = 1 here
    assert np.array_equal(xt_r, (x * m.astype(np.float32)).astype(np.float32))


def test_pack_lists_distinct_columns_with_weighted_values():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 120)).astype(np.float32)
    for scheme in (R.REPLACE_SHARED, R.REPLACE_PER_EXAMPLE):
        rp, col, val, xt = R.sample_pack(x, scheme, 0.3, 8, 2, 1)
        m = R.multiplicity(scheme, 0.3, 8, 2, 1, 5, 120)
        k = R.fixed_k(0.3, 120)
        scale = np.float32(120 / k)
        for b in range(5):
            cols = col[rp[b]:rp[b + 1]]
            assert np.array_equal(cols, np.nonzero(m[b])[0])          # ascending, each once
            w = (m[b, cols].astype(np.float32) * scale).astype(np.float32)
            assert np.array_equal(val[rp[b]:rp[b + 1]], (x[b, cols] * w).astype(np.float32))
        assert np.array_equal(xt != 0, (m > 0) & (x != 0))


@pytest.mark.parametrize("scheme", [R.REPLACE_PER_EXAMPLE, R.REPLACE_SHARED])
def test_unbiased_and_variance_closed_form(scheme):
    """E[P] = I (Section 3.2).  Var m_j = k (1/d)(1 - 1/d), so with independent rows
    Var dW~[j,n] = ((d-1)/k) sum_b x[b,j]^2 g[b,n]^2, and with one shared set ((d-1)/k) dW[j,n]^2."""
    rng = np.random.default_rng(13)
    B, D, N, p, S = 10, 40, 4, 0.25, 6000
    x = rng.standard_normal((B, D)).astype(np.float32)
    dy = rng.standard_normal((B, N)).astype(np.float32)
    bits = rng.random((B, N)) > 0.4
    g = dy.astype(np.float64) * bits
    exact = x.astype(np.float64).T @ g
    acc = np.zeros_like(exact)
    acc2 = np.zeros_like(exact)
    for s in range(S):
        e = R.backward_dW(R.sample_pack(x, scheme, p, s, 1, 0)[3], dy, bits)
        acc += e
        acc2 += e * e
    mean = acc / S
    var = acc2 / S - mean**2
    k = R.fixed_k(p, D)
    if scheme == R.REPLACE_SHARED:
        var_cf = (D - 1) / k * exact**2
    else:
        var_cf = (D - 1) / k * (x.astype(np.float64) ** 2).T @ g**2
    err = np.linalg.norm(mean - exact)
    assert 0 < err < 4 * np.sqrt(var_cf.sum() / S)
    assert abs(var.sum() / var_cf.sum() - 1) < 0.08
    # more variance than the draw without replacement at the same k, whose factor is d/k - 1 instead
    var_without = var_cf * (D / k - 1) / ((D - 1) / k)
    assert var.sum() > 1.15 * var_without.sum()


def test_train_step_runs_and_keeps_the_exact_chain():
    rng = np.random.default_rng(4)
    dims = [20, 16, 12, 5]
    x = rng.standard_normal((10, 20)).astype(np.float32)
    Ws = [(rng.standard_normal((dims[i], dims[i + 1])) / np.sqrt(dims[i])).astype(np.float32) for i in range(3)]
    bs = [np.zeros(dims[i + 1], np.float32) for i in range(3)]
    labels = rng.integers(0, 5, 10).astype(np.int32)
    ref = R.mlp_train_step(x, labels, Ws, bs, R.EXACT, 1.0, seed=0)
    for scheme in (R.REPLACE_SHARED, R.REPLACE_PER_EXAMPLE):
        out = R.mlp_train_step(x, labels, Ws, bs, scheme, 0.3, seed=2)
        assert out["loss"] == ref["loss"]
        for l in range(3):
            assert np.array_equal(out["dy"][l], ref["dy"][l])          # dX chain never sees a sample
            assert not np.array_equal(out["dW"][l], ref["dW"][l])

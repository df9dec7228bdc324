"""Pins for the selection rules, the scale and the byte accounting of the
oracle: the paper's worked values, brute force on tiny inputs, and the
distributional facts the definition of P (Section 3.2) fixes."""
import os

import numpy as np
import pytest

from oracle import rad_oracle as R

GOLD = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden")


def _rows(name):
    with open(os.path.join(GOLD, name)) as fh:
        return [ln.split() for ln in fh if ln.strip() and not ln.startswith("#")]


def test_fixed_k_worked_values():
    for p, d, k in _rows("appendix_a_k_values.txt"):
        assert R.fixed_k(float(p), int(d)) == int(k)


def test_fixed_k_limits():
    assert R.fixed_k(1.0, 784) == 784
    assert R.fixed_k(1e-9, 784) == 1
    assert R.fixed_k(0.5, 4096) == 2048 and R.fixed_k(0.02, 4096) == 82
    for d in (1, 7, 300, 4096):
        for p in (0.01, 0.1, 0.3, 0.5, 0.99, 1.0):
            k = R.fixed_k(p, d)
            assert 1 <= k <= d and k >= p * d - 1e-6 and k < p * d + 1


FC = dict(dims=[784, 300, 300, 300], logits=10, relu=900,
          params=784 * 300 + 300 + 2 * (300 * 300 + 300) + 300 * 10 + 10)
CONV = dict(dims=[3072, 16384, 8192, 8192, 2048], logits=10,
            relu=16384 + 8192 + 8192 + 2048,
            params=(3 * 25 * 16 + 16) + (16 * 25 * 32 + 32) + 2 * (32 * 25 * 32 + 32)
            + 2048 * 10 + 10)
RNN = dict(dims=[1, 100] * 784 + [100], logits=10, relu=784 * 100,
           params=100 + 100 + 100 * 100 + 100 + 100 * 10 + 10)
NETS = dict(fc=FC, conv=CONV, rnn=RNN)


def test_appendix_a_bytes_per_example():
    for name, base, rad in _rows("appendix_a_bytes.txt"):
        n = NETS[name]
        assert R.paper_bytes_per_example(n["dims"], n["logits"], n["relu"], 1.0) == float(base)
        assert R.paper_bytes_per_example(n["dims"], n["logits"], n["relu"], 0.1) == float(rad)


def test_table1_total_memory():
    rows = _rows("table1_peak_memory_mb.txt")
    fr = [float(v) for v in rows[0][1:]]
    for row in rows[1:]:
        n = NETS[row[0]]
        offset = 0.31 if row[0] == "rnn" else 0.0    # see the fixture's header
        for p, printed in zip(fr, row[1:]):
            got = R.paper_total_megabytes(n["params"], 150, n["dims"], n["logits"], n["relu"], p)
            assert abs(got + offset - float(printed)) <= 0.0101, (row[0], p, got)


def test_bernoulli_threshold():
    assert R.bernoulli_threshold(1.0) == 1 << 32
    assert R.bernoulli_threshold(0.5) == 1 << 31
    assert R.bernoulli_threshold(0.1) == 429496730
    m = R.keep_mask(R.BERNOULLI, 1.0, 5, 0, 0, 7, 33)
    assert m.all()


def test_fixed_k_brute_force_with_ties():
    # keys recomputed here; selection by python's sort on (key, j) tuples
    for seed, rows, d, p in [(1, 5, 13, 0.3), (2, 3, 64, 0.1), (3, 4, 7, 1.0)]:
        k = R.fixed_k(p, d)
        keys = R.element_keys(seed, 4, 9, 0, rows * d).reshape(rows, d)
        m = R.keep_mask(R.FIXEDK_PER_EXAMPLE, p, seed, 4, 9, rows, d)
        for b in range(rows):
            want = sorted(j for _, j in sorted((int(keys[b, j]), j) for j in range(d))[:k])
            assert list(np.nonzero(m[b])[0]) == want
    # a forced tie: the stable order must take the lower index
    keys = np.array([[5, 3, 3, 9, 3]], dtype=np.uint32)
    order = np.argsort(keys, axis=1, kind="stable")
    assert list(order[0, :2]) == [1, 2]


def test_shared_scheme_is_one_row_of_keys():
    m = R.keep_mask(R.FIXEDK_SHARED, 0.1, 11, 2, 0, 6, 300)
    assert (m == m[0]).all() and m[0].sum() == 30
    keys = R.element_keys(11, 2, 0, 0, 300)
    assert set(np.nonzero(m[0])[0]) == set(np.argsort(keys, kind="stable")[:30])


def test_store_sizes():
    x = np.ones((150, 784), dtype=np.float32)
    rp, col, val, xt = R.sample_pack(x, R.FIXEDK_PER_EXAMPLE, 0.1, 3, 0, 0)
    assert rp[-1] == 150 * 79 and (np.diff(rp) == 79).all()
    assert np.all(val == np.float32(784 / 79))
    rp, col, val, xt = R.sample_pack(x, R.BERNOULLI, 0.1, 3, 0, 0)
    n = 150 * 784
    assert abs(rp[-1] - 0.1 * n) < 5 * np.sqrt(n * 0.1 * 0.9)      # nnz ~ Binomial
    assert np.all(val == np.float32(10.0))
    for b in range(0, 150, 37):                                    # ascending columns
        c = col[rp[b]:rp[b + 1]]
        assert np.all(np.diff(c) > 0)
        assert np.all(xt[b, c] == val[rp[b]:rp[b + 1]])
    rp, col, val, xt = R.sample_pack(x, R.EXACT, 0.1, 3, 0, 0)
    assert rp[-1] == n and np.array_equal(xt, x)


def test_inclusion_frequency_and_independence():
    d, k, trials = 64, 7, 4000
    cnt = np.zeros(d)
    overlap = 0.0
    for s in range(trials):
        m = R.keep_mask(R.FIXEDK_PER_EXAMPLE, k / d, s, 0, 0, 2, d)
        cnt += m[0]
        overlap += (m[0] & m[1]).sum()
    pi = k / d
    z = (cnt / trials - pi) / np.sqrt(pi * (1 - pi) / trials)
    assert np.abs(z).max() < 4.5                   # every coordinate equally likely
    # two examples draw independent subsets: E|S1 n S2| = k^2/d
    assert abs(overlap / trials - k * k / d) < 5 * np.sqrt(k * k / d / trials)


def test_scale():
    assert R.sample_scale(R.BERNOULLI, 0.1, 784) == np.float32(10.0)
    assert R.sample_scale(R.FIXEDK_SHARED, 0.1, 784) == np.float32(784 / 79)
    assert R.sample_scale(R.FIXEDK_PER_EXAMPLE, 1.0, 300) == np.float32(1.0)


def test_round_bf16_equals_torch_cast():
    import torch
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(100000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 100000),
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, np.inf, -np.inf, 3.3895314e38], dtype=np.float32)])
    want = torch.from_numpy(a).to(torch.bfloat16).to(torch.float32).numpy()
    got = R.round_bf16(a)
    assert np.array_equal(got.view(np.uint32), want.view(np.uint32))

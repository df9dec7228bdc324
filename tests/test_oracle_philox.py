"""Pins the oracle's Philox4x32-10 to PyTorch's own CPU engine
(ATen/core/PhiloxRNGEngine.h), compiled here into a tiny probe: an
implementation the oracle shares nothing with."""
import os
import subprocess
import sys

import numpy as np
import pytest

from oracle import rad_oracle as R

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def probe(tmp_path_factory):
    import torch
    inc = os.path.join(os.path.dirname(torch.__file__), "include")
    exe = str(tmp_path_factory.mktemp("philox") / "aten_philox_probe")
    subprocess.check_call(["g++", "-O1", "-std=c++17", "-I" + inc,
                           os.path.join(HERE, "aten_philox_probe.cpp"), "-o", exe])
    return exe


def aten_words(exe, seed, stream_id, step, first_quad, n_words):
    sub = (step << 32) | stream_id
    out = subprocess.check_output([exe, str(seed), str(sub), str(first_quad), str(n_words)])
    return np.array([int(t) for t in out.split()], dtype=np.uint32)


@pytest.mark.parametrize("seed,stream_id,step,first_quad", [
    (0, 0, 0, 0),
    (1234, 0, 0, 0),
    (0xDEADBEEFCAFEF00D, 7, 3, 12345),
    (42, 0xF0000001, 783, (1 << 32) + 5),      # counter word 1 in use
    ((1 << 64) - 1, 0xFFFFFFFF, 0xFFFFFFFF, (1 << 40)),
])
def test_keys_equal_aten_engine(probe, seed, stream_id, step, first_quad):
    n = 4096
    want = aten_words(probe, seed, stream_id, step, first_quad, n)
    got = R.element_keys(seed, stream_id, step, 4 * first_quad, n)
    assert np.array_equal(got, want)


def test_unaligned_first_element(probe):
    want = aten_words(probe, 99, 2, 5, 10, 64)
    got = R.element_keys(99, 2, 5, 43, 17)         # f = 43 = quad 10, word 3
    assert np.array_equal(got, want[3:20])


def test_key_statistics():
    k = R.element_keys(2024, 1, 0, 0, 1 << 20)
    u = k.astype(np.float64) / 2.0**32
    n = u.size
    assert abs(u.mean() - 0.5) < 5 * np.sqrt(1 / 12 / n)
    bits = ((k[:, None] >> np.arange(32, dtype=np.uint32)) & 1).mean(axis=0)
    assert np.all(np.abs(bits - 0.5) < 5 * 0.5 / np.sqrt(n))
    # distinct streams / steps / seeds give unrelated keys
    for other in (R.element_keys(2024, 2, 0, 0, 1 << 12),
                  R.element_keys(2024, 1, 1, 0, 1 << 12),
                  R.element_keys(2025, 1, 0, 0, 1 << 12)):
        assert (other == k[:1 << 12]).mean() < 0.01

"""The gradient-noise procedure (Section 4.3, gradient-noise figure) run through the C ABI against the same
procedure run on the oracle's training steps: per-layer mean squared deviations of every method agree, and
they order as the paper reports (sampling costs less noise than the reduced minibatch of equal memory)."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import rad_oracle as R


def test_small_mlp_matches_the_oracle_procedure():
    from paper_2007_10412_amd import gradient_noise as G
    cfg = dict(kind="mlp", dims=(64, 48, 32, 10), batch=24, reduced=4)
    data = G.training_set(cfg, 96, seed=3)
    methods = G.methods_for(cfg, 0.25)
    L = len(cfg["dims"]) - 1

    def oracle_step(first, count, scheme, p, seed):
        out = R.mlp_train_step(data["x"][first:first + count], data["labels"][first:first + count], data["Ws"], data["bs"],
                               scheme, p, seed)
        return out["dW"]
    want = G.measure(oracle_step, 96, methods, draws=6)
    step = G.GpuStep(cfg, data)
    try:
        got = G.measure(step, 96, methods, draws=6)
    finally:
        step.close()
    print(got, flush=True)
    for name in methods:
        assert np.allclose(got[name], want[name], rtol=2e-3), (name, got[name], want[name])
    # a reduced minibatch is noisier than sampling a quarter of the activations of the whole minibatch
    for l in range(L):
        assert got["different_sample"][l] < got["reduced_batch"][l]
        assert got["baseline"][l] <= got["different_sample"][l]
        assert got["different_sample_2x_batch"][l] < got["different_sample"][l]


def test_paper_convnet_runs():
    """The convolutional architecture of Appendix A on a 300-example synthetic set: finite numbers for every
    method and layer, baseline below reduced batch."""
    from paper_2007_10412_amd import gradient_noise as G
    cfg = G.paper_arch("cnn")
    step = G.GpuStep(cfg, G.training_set(cfg, 300))
    try:
        got = G.measure(step, 300, G.methods_for(cfg, 0.1), draws=3)
    finally:
        step.close()
    print(got, flush=True)
    for name, v in got.items():
        assert len(v) == 5 and np.all(np.isfinite(v)), name
    assert all(a < b for a, b in zip(got["baseline"], got["reduced_batch"]))


def test_small_rnn_matches_the_oracle_procedure():
    """The recurrent leg (input, recurrent and output weights as the three "layers"; Appendix A's reduced
    minibatch is 21 of 150, here 3 of 16) on a short sequence against the oracle's BPTT."""
    from paper_2007_10412_amd import gradient_noise as G
    cfg = dict(kind="rnn", T=12, d_input=1, hidden=32, classes=10, batch=16, reduced=3)
    data = G.training_set(cfg, 48, seed=5)
    methods = G.methods_for(cfg, 0.25)

    def oracle_step(first, count, scheme, p, seed):
        sl = slice(first, first + count)
        out = R.rnn_train_step(data["x"][sl], data["labels"][sl], data["W_ih"], data["W_hh"], data["b"], data["W_ho"],
                               data["b_o"], scheme, p, seed)
        return [out["dW_ih"], out["dW_hh"], out["dW_ho"]]
    want = G.measure(oracle_step, 48, methods, draws=5)
    step = G.GpuStep(cfg, data)
    try:
        got = G.measure(step, 48, methods, draws=5)
    finally:
        step.close()
    print(got, flush=True)
    for name in methods:
        assert np.allclose(got[name], want[name], rtol=2e-3), (name, got[name], want[name])
    assert got["baseline"][1] <= got["different_sample"][1] < got["reduced_batch"][1]


def test_paper_rnn_runs():
    """The recurrent architecture of Appendix A (784 steps, hidden 100, minibatch 150, reduced minibatch 21) on a
    300-example synthetic set: finite numbers for every method."""
    from paper_2007_10412_amd import gradient_noise as G
    cfg = G.paper_arch("rnn")
    step = G.GpuStep(cfg, G.training_set(cfg, 300))
    try:
        got = G.measure(step, 300, G.methods_for(cfg, 0.1), draws=2)
    finally:
        step.close()
    print(got, flush=True)
    for name, v in got.items():
        assert len(v) == 3 and np.all(np.isfinite(v)), name

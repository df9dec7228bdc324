"""GPU parity of rad_train_step on the ReLU RNN (config 5): forward, BPTT from
per-step sampled hidden states, every gradient against the oracle."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import rad_oracle as R


@pytest.fixture(scope="module")
def ctx():
    from paper_2007_10412_amd import binding as B
    c = B.rad_ctx_create()
    yield c
    B.rad_ctx_destroy(c)


def run_rnn(ctx, d, scheme, p, seed, check_store=True):
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty, rel_err, assert_grad_close, U_F32
    Bt, T, I = d["x"].shape
    H, C = d["W_ho"].shape
    print("rnn B=%d T=%d I=%d H=%d scheme=%d p=%g" % (Bt, T, I, H, scheme, p), flush=True)
    m = B.rad_model_create_rnn(ctx, Bt, T, I, H, C, scheme, p)
    try:
        names = ["W_ih", "W_hh", "b", "W_ho", "b_o"]
        params = [dev(d[n]) for n in names]
        grads = [empty(d[n].shape) for n in names]
        loss = B.rad_train_step(ctx, m, B.make_sampling(scheme, p, seed, 20, 0), dev(d["x"]), dev(d["labels"]),
                                params, grads)
        ref = R.rnn_train_step(d["x"], d["labels"], d["W_ih"], d["W_hh"], d["b"], d["W_ho"], d["b_o"],
                               scheme, p, seed, stream_base=20)
        assert abs(loss - ref["loss"]) < 1e-5 * max(1.0, abs(ref["loss"])), (loss, ref["loss"])
        if check_store and scheme != 0 and T > 1:
            # sampling decisions of every step: rows t*B..(t+1)*B-1 of the multi-step store hold step t+2
            # every row of every step: the column lists exactly, the values within fp32 rounding of the hidden state
            rp, col, val = B.rad_store_export_csr(ctx, B.rad_model_store(m, 0), (T - 1) * Bt)
            steps = ref["stores"][2:]
            want_rp = np.concatenate([[0], np.cumsum(np.concatenate([np.diff(s[0]) for s in steps]))])
            assert np.array_equal(rp, want_rp)
            assert np.array_equal(col, np.concatenate([s[1] for s in steps]))
            want_val = np.concatenate([s[2] for s in steps]).astype(np.float64)
            assert np.abs(val - want_val).max() <= 1e-5 * max(1.0, np.abs(want_val).max())
            rp, col, val = B.rad_store_export_csr(ctx, B.rad_model_store(m, 1), Bt)
            assert np.array_equal(rp, ref["store_o"][0]) and np.array_equal(col, ref["store_o"][1])
            assert np.abs(val - ref["store_o"][2]).max() <= 1e-5 * max(1.0, np.abs(ref["store_o"][2]).max())
        out = {}
        # contraction lengths: the recurrent gradients sum over steps x batch
        for n, key, K in zip(names, ["dW_ih", "dW_hh", "db", "dW_ho", "db_o"], [T * Bt, T * Bt, T * Bt, Bt, Bt]):
            out[key] = assert_grad_close(host(grads[names.index(n)]), ref[key], 1e-4, K, key, acc_u=U_F32, c=32.0)[0]
        return out
    finally:
        B.rad_model_destroy(m)


@pytest.mark.parametrize("scheme,p", [(1, 0.1), (3, 0.25), (2, 0.25), (0, 1.0), (1, 1.0)])
def test_rnn_small_general_weights(ctx, scheme, p):
    from paper_2007_10412_amd import synth
    d = synth.rnn(seed=3, batch=20, T=9, d_input=1, hidden=96, classes=10, identity=False)
    run_rnn(ctx, d, scheme, p, seed=8)


def test_rnn_two_inputs_ragged(ctx):
    from paper_2007_10412_amd import synth
    d = synth.rnn(seed=4, batch=7, T=5, d_input=2, hidden=70, classes=6, identity=False)
    run_rnn(ctx, d, 1, 0.3, seed=2)


def test_rnn_single_step(ctx):
    from paper_2007_10412_amd import synth
    d = synth.rnn(seed=5, batch=9, T=1, d_input=1, hidden=64, classes=10, identity=False)
    run_rnn(ctx, d, 1, 0.5, seed=2, check_store=False)


def test_config5_reduced_length(ctx):
    """Config 5's widths (batch 128, hidden 1024, identity W_hh) with T = 48: the oracle's 784-step
    BPTT in fp64 takes minutes, the structure of every step is the same."""
    from paper_2007_10412_amd import synth
    d = synth.rnn(seed=1234, batch=128, T=48, d_input=1, hidden=1024, classes=10, identity=True)
    run_rnn(ctx, d, 1, 0.1, seed=5)


@pytest.mark.parametrize("scheme", [2, 3])
def test_paper_rnn_widths(ctx, scheme):
    """The recurrent architecture of Appendix A (hidden state 100, one-dimensional input, minibatch 150,
    identity recurrent weights) over 40 time steps, "same sample" and "different sample" at fraction 0.1."""
    from paper_2007_10412_amd import synth
    d = synth.rnn(seed=77, batch=150, T=40, d_input=1, hidden=100, classes=10, identity=True)
    run_rnn(ctx, d, scheme, 0.1, seed=9)


@pytest.mark.parametrize("T", [2, 10, 17])
@pytest.mark.parametrize("scheme,p", [(1, 0.3), (3, 0.25), (0, 1.0), (2, 0.25)])
def test_rnn_lengths_around_the_chunks_of_the_recurrent_dW(ctx, T, scheme, p):
    """The recurrent dW, the bias gradient and the input-weight gradient are formed over chunks of eight time
    steps (T - 1 = 1: a single short chunk; 9: one whole chunk and one step; 16: two whole chunks); the shared
    scheme keeps the step-by-step form.  Every gradient against the oracle."""
    from paper_2007_10412_amd import synth
    d = synth.rnn(seed=20 + T, batch=8, T=T, d_input=2, hidden=64, classes=5, identity=False)
    run_rnn(ctx, d, scheme, p, seed=T)


def test_rnn_hidden_width_whose_split_ranges_need_rounding(ctx):
    """Hidden width 576 with whole 64 x 64 tiles: the per-step forward and dX GEMMs take the unguarded split-K
    kernels, whose K ranges must be whole 32-deep slices (576 / 4 = 144 is not)."""
    from paper_2007_10412_amd import synth
    d = synth.rnn(seed=6, batch=64, T=6, d_input=1, hidden=576, classes=10, identity=False)
    run_rnn(ctx, d, 1, 0.2, seed=3)


@pytest.mark.parametrize("scheme", [6, 7])
@pytest.mark.parametrize("T", [1, 7])
def test_rnn_random_projections(ctx, scheme, T):
    """"project" and "different project" of the recurrent experiments (Appendix A, RNN training details): every
    step stores z_t = h_{t-1} R_t / sqrt(k) with a sign matrix drawn afresh per step (one per example for scheme
    7), and dW_hh is formed from z_t and the regenerated R_t."""
    from paper_2007_10412_amd import synth
    d = synth.rnn(seed=30 + T, batch=8, T=T, d_input=1, hidden=64, classes=10, identity=False)
    run_rnn(ctx, d, scheme, 0.25, seed=5)


def test_paper_rnn_widths_projected(ctx):
    from paper_2007_10412_amd import synth
    d = synth.rnn(seed=78, batch=150, T=12, d_input=1, hidden=100, classes=10, identity=True)
    run_rnn(ctx, d, 6, 0.1, seed=9)

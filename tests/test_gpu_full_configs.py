"""Parity at the full sizes of the five configurations, in the launch
configuration bench.py times (config 4) — the oracle finishes each in well
under a minute, so every output is compared, not a sample."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2007_10412_amd import binding as B
    c = B.rad_ctx_create()
    yield c
    B.rad_ctx_destroy(c)


def test_config3_full(ctx):
    from paper_2007_10412_amd import synth
    from tests.test_gpu_cnn import run_cnn
    ch, pool = (3, 16, 32, 64), (0, 1, 1)
    d = synth.cnn(seed=1234, batch=150, channels=ch, pool=pool, ksize=3, hw=32, classes=10)
    flips, swaps = run_cnn(ctx, d, ch, pool, 3, 32, 10, 1, 0.1, seed=5)
    print("config 3: %d ReLU-bit flips, %d pool swaps taken from the GPU" % (flips, swaps))


@pytest.mark.parametrize("scheme", [3, 2])
@pytest.mark.parametrize("p", [0.5, 0.1, 0.02])
def test_config4_full(ctx, scheme, p):
    """All six fraction x scheme variants of the wide bf16 MLP at full size."""
    from paper_2007_10412_amd import binding as B, synth
    from tests.test_gpu_mlp import run_mlp
    dims = (4096, 4096, 4096, 1000)
    data = synth.mlp(seed=1234, batch=4096, dims=dims, pixels=False, bf16=True)
    run_mlp(ctx, data, dims, scheme, p, seed=1000, dtype=B.RAD_BF16, has_bias=False)


def test_config4_full_with_biases(ctx):
    """The same network with biases (per-example fixed-k, fraction 0.1): the bias gradients are column sums of the
    loss gradient, which this model keeps with rows padded to 1024 for its 1000-wide last layer."""
    from paper_2007_10412_amd import binding as B, synth
    from tests.test_gpu_mlp import run_mlp
    dims = (4096, 4096, 4096, 1000)
    data = synth.mlp(seed=4321, batch=4096, dims=dims, pixels=False, bf16=True, bias_scale=0.1)
    run_mlp(ctx, data, dims, 3, 0.1, seed=1001, dtype=B.RAD_BF16, has_bias=True)


def test_config5_full(ctx):
    from paper_2007_10412_amd import synth
    from tests.test_gpu_rnn import run_rnn
    d = synth.rnn(seed=1234, batch=128, T=784, d_input=1, hidden=1024, classes=10, identity=True)
    run_rnn(ctx, d, 1, 0.1, seed=5)

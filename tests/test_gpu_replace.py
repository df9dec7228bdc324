"""GPU parity of the with-replacement sampling schemes (Section 3.2, the matrix P as printed): stores
bit-exact against the oracle (columns, draw-count weights, values), gradients within tolerance."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import rad_oracle as R
from tests.test_gpu_sampling import _check_pack
from tests.test_gpu_linear import run_layer
from tests.test_gpu_mlp import run_mlp


@pytest.fixture(scope="module")
def ctx():
    from paper_2007_10412_amd import binding as B
    c = B.rad_ctx_create()
    yield c
    B.rad_ctx_destroy(c)


@pytest.mark.parametrize("scheme", [4, 5])
@pytest.mark.parametrize("rows,cols,p", [
    (150, 784, 0.1),
    (150, 300, 0.1),
    (33, 37, 0.3),          # rows start inside a Philox call (k % 4 != 0), one ragged bucket
    (5, 1, 0.1),            # one column: drawn once
    (3, 1030, 0.5),
    (64, 4096, 0.02),
    (2, 16384, 0.1),        # widest row
    (7, 300, 1.0),          # full fraction: k = d draws, columns repeat and others are missing
])
def test_pack_equals_oracle_f32(ctx, scheme, rows, cols, p):
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(rows * 1000 + cols)
    _check_pack(ctx, rows, cols, scheme, p, seed=31 + rows, stream_id=3, step=5, dtype=B.RAD_F32, rng=rng)


@pytest.mark.parametrize("scheme", [4, 5])
def test_pack_equals_oracle_bf16(ctx, scheme):
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(5)
    _check_pack(ctx, 96, 4096, scheme, 0.1, seed=(1 << 40) + 9, stream_id=1, step=0, dtype=B.RAD_BF16, rng=rng)


def test_full_fraction_differs_from_without_replacement(ctx):
    """Appendix A, fraction sweep: with replacement the full fraction is not the baseline."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev
    x = np.arange(1, 8 * 64 + 1, dtype=np.float32).reshape(8, 64)
    out = {}
    for scheme in (3, 5):
        st = B.rad_store_create(ctx, B.make_layer(8, 64, 8, relu=False), scheme, 1.0)
        try:
            B.rad_sample_pack(ctx, B.make_sampling(scheme, 1.0, 7, 0, 0), dev(x), st)
            out[scheme] = B.rad_store_export_csr(ctx, st, 8)
        finally:
            B.rad_store_destroy(st)
    assert out[3][0][-1] == 8 * 64 and np.array_equal(out[3][2], x.ravel())
    assert out[5][0][-1] < 8 * 64                           # some columns were never drawn
    assert out[5][2].sum() == pytest.approx(x.sum(), rel=0.2) and not np.array_equal(out[5][2], out[3][2][: len(out[5][2])])


@pytest.mark.parametrize("scheme", [4, 5])
@pytest.mark.parametrize("Bt,D,N", [(7, 37, 10), (150, 784, 300), (130, 260, 70)])
def test_layer_f32(ctx, scheme, Bt, D, N):
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(Bt * 7 + D)
    x = rng.standard_normal((Bt, D)).astype(np.float32)
    W = (rng.standard_normal((D, N)) / np.sqrt(D)).astype(np.float32)
    bias = (0.1 * rng.standard_normal(N)).astype(np.float32)
    dy = rng.standard_normal((Bt, N)).astype(np.float32)
    run_layer(ctx, x, W, bias, dy, scheme, 0.3, seed=5, dtype=B.RAD_F32)


@pytest.mark.parametrize("scheme,p", [(5, 0.1), (4, 0.1), (5, 0.5), (5, 0.02)])
def test_layer_bf16(ctx, scheme, p):
    from paper_2007_10412_amd import binding as B
    from paper_2007_10412_amd.synth import bf16_round
    rng = np.random.default_rng(4)
    Bt, D, N = 512, 1024, 768
    x = bf16_round(rng.standard_normal((Bt, D)))
    W = bf16_round(rng.standard_normal((D, N)) / np.sqrt(D))
    dy = bf16_round(rng.standard_normal((Bt, N)) * 0.01)
    run_layer(ctx, x, W, None, dy, scheme, p, seed=12, dtype=B.RAD_BF16)


@pytest.mark.parametrize("scheme", [4, 5])
def test_mlp_f32(ctx, scheme):
    from paper_2007_10412_amd import binding as B, synth
    data = synth.mlp(seed=1234, batch=150, dims=(784, 300, 300, 10), bias_scale=0.0)
    run_mlp(ctx, data, (784, 300, 300, 10), scheme, 0.1, seed=42, dtype=B.RAD_F32, has_bias=True)


@pytest.mark.parametrize("scheme,p", [(5, 0.1), (4, 0.1), (5, 0.5)])
def test_mlp_bf16_reduced(ctx, scheme, p):
    """Config 4's structure at a size the oracle finishes in seconds; the epilogue packs with draw-count weights."""
    from paper_2007_10412_amd import binding as B, synth
    dims = (1024, 768, 512, 1000)
    data = synth.mlp(seed=3, batch=512, dims=dims, pixels=False, bf16=True)
    run_mlp(ctx, data, dims, scheme, p, seed=6, dtype=B.RAD_BF16, has_bias=False)


def test_unbiased_over_seeds(ctx):
    """E[P] = I on the GPU path: the mean of dW over seeds approaches the exact dW at the closed-form rate."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty
    rng = np.random.default_rng(8)
    Bt, D, N, p, S = 32, 96, 16, 0.25, 400
    x = rng.standard_normal((Bt, D)).astype(np.float32)
    dy = rng.standard_normal((Bt, N)).astype(np.float32)
    exact = x.astype(np.float64).T @ dy.astype(np.float64)
    L = B.make_layer(Bt, D, N, relu=False)
    st = B.rad_store_create(ctx, L, 5, p)
    try:
        gx, gdy, gW = dev(x), dev(dy), empty((D, N))
        acc = np.zeros_like(exact)
        for s in range(S):
            B.rad_sample_pack(ctx, B.make_sampling(5, p, s, 0, 0), gx, st)
            B.rad_backward_dW(ctx, L, st, gdy, gW, None, 0.0)
            acc += host(gW)
    finally:
        B.rad_store_destroy(st)
    k = R.fixed_k(p, D)
    var_cf = (D - 1) / k * (x.astype(np.float64) ** 2).T @ dy.astype(np.float64) ** 2
    err = np.linalg.norm(acc / S - exact)
    assert 0 < err < 4 * np.sqrt(var_cf.sum() / S)


@pytest.mark.parametrize("scheme", [4, 5])
def test_cnn_small(ctx, scheme):
    from paper_2007_10412_amd import synth
    from tests.test_gpu_cnn import run_cnn
    ch, pool = (3, 8, 12, 16), (0, 1, 1)
    d = synth.cnn(seed=7, batch=6, channels=ch, pool=pool, ksize=3, hw=16, classes=10)
    run_cnn(ctx, d, ch, pool, 3, 16, 10, scheme, 0.25, seed=3)


@pytest.mark.parametrize("scheme", [4, 5])
def test_rnn_small(ctx, scheme):
    """A multi-step store: the draw counts of every time step are written by one plan launch."""
    from paper_2007_10412_amd import synth
    from tests.test_gpu_rnn import run_rnn
    d = synth.rnn(seed=3, batch=20, T=9, d_input=1, hidden=96, classes=10, identity=False)
    run_rnn(ctx, d, scheme, 0.25, seed=8)


def test_config4_full_with_replacement(ctx):
    """Config 4 at full size with the paper's own draw, every output compared."""
    from paper_2007_10412_amd import binding as B, synth
    dims = (4096, 4096, 4096, 1000)
    data = synth.mlp(seed=1234, batch=4096, dims=dims, pixels=False, bf16=True)
    run_mlp(ctx, data, dims, 5, 0.1, seed=1000, dtype=B.RAD_BF16, has_bias=False)

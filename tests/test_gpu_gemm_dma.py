"""GPU parity of the bf16 GEMM kernels that load global memory straight into LDS: wide interior shapes of
rad_forward_sample (K-contiguous x, M/N-contiguous W read through transposing LDS reads) and of
rad_backward_dX (two K-contiguous operands) against the oracle, over contraction lengths that end the
pipeline at every point: one slice, odd and even slice counts, whole and ragged last slices."""
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


def bf16_data(rng, shape, scale=1.0):
    # values exactly representable in bf16, so that both sides start from the same numbers
    return R.round_bf16((rng.standard_normal(shape) * scale).astype(np.float32))


@pytest.mark.parametrize("d_in", [8, 40, 64, 128, 192, 200, 320, 1024])
@pytest.mark.parametrize("relu", [False, True])
def test_forward_wide_layer(ctx, d_in, relu):
    """128 output tiles of 256 x 256: y, and the ReLU bits, of a 2048 x d_in x 4096 layer."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty, unpack_bits, rel_err, assert_bits_match, TOL
    Bt, N = 2048, 4096
    rng = np.random.default_rng(100 + d_in)
    x = bf16_data(rng, (Bt, d_in))
    W = bf16_data(rng, (d_in, N), 1.0 / np.sqrt(d_in))
    bias = rng.standard_normal(N).astype(np.float32)
    print("forward B=%d D=%d N=%d relu=%d" % (Bt, d_in, N, relu), flush=True)
    L = B.make_layer(Bt, d_in, N, dtype=B.RAD_BF16, relu=relu, has_bias=True)
    st = B.rad_store_create(ctx, L, B.RAD_FIXEDK_PER_EXAMPLE, 0.25)
    try:
        y = empty((Bt, N), B.RAD_BF16)
        B.rad_forward_sample(ctx, L, B.make_sampling(B.RAD_FIXEDK_PER_EXAMPLE, 0.25, 7), dev(x, B.RAD_BF16),
                             dev(W, B.RAD_BF16), dev(bias), y, st)
        h, oy, _ = R.linear_forward(x, W, bias, relu, B.RAD_BF16)
        assert rel_err(host(y), oy) < TOL[B.RAD_BF16]
        # element by element: bf16 rounding of an fp32 sum of d_in products
        assert np.max(np.abs(host(y) - oy)) <= 2.0 ** -7 * max(1.0, np.max(np.abs(oy)))
        if relu:
            bits = unpack_bits(B.rad_store_export_bits(ctx, st, Bt, N), N)
            assert_bits_match(bits, h, "relu bits")
    finally:
        B.rad_store_destroy(st)


@pytest.mark.parametrize("d_out", [8, 32, 40, 64, 96, 128, 160, 192, 256, 288, 448, 1000])
def test_dX_wide_layer(ctx, d_out):
    """128 output tiles of 256 x 256: dX = dy W^T for a 2048 x 4096 x d_out layer without ReLU."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty, rel_err, TOL
    Bt, D = 2048, 4096
    rng = np.random.default_rng(200 + d_out)
    dy = bf16_data(rng, (Bt, d_out))
    W = bf16_data(rng, (D, d_out), 1.0 / np.sqrt(d_out))
    print("dX B=%d D=%d N=%d" % (Bt, D, d_out), flush=True)
    L = B.make_layer(Bt, D, d_out, dtype=B.RAD_BF16, relu=False)
    st = B.rad_store_create(ctx, L, B.RAD_FIXEDK_PER_EXAMPLE, 0.1)
    try:
        dX = empty((Bt, D), B.RAD_BF16)
        B.rad_backward_dX(ctx, L, st, dev(dy, B.RAD_BF16), dev(W, B.RAD_BF16), dX)
        want = R.backward_dX(dy, np.ones((Bt, d_out), dtype=bool), W)
        assert rel_err(host(dX), want) < TOL[B.RAD_BF16]
        assert np.max(np.abs(host(dX) - want)) <= 2.0 ** -7 * max(1.0, np.max(np.abs(want)))
    finally:
        B.rad_store_destroy(st)


@pytest.mark.parametrize("batch", [8, 64, 72, 128, 192, 200, 320, 1024])
def test_dense_dW_wide_layer(ctx, batch):
    """128 output tiles of 256 x 256: dW = x^T dy from an exact store (both operands M/N contiguous), and
    its accumulating form."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty, rel_err, TOL
    D, N = 2048, 4096
    rng = np.random.default_rng(300 + batch)
    x = bf16_data(rng, (batch, D))
    dy = bf16_data(rng, (batch, N))
    W = bf16_data(rng, (D, N), 1.0 / 64)
    print("dense dW B=%d D=%d N=%d" % (batch, D, N), flush=True)
    L = B.make_layer(batch, D, N, dtype=B.RAD_BF16, relu=False)
    st = B.rad_store_create(ctx, L, B.RAD_EXACT, 1.0)
    try:
        y = empty((batch, N), B.RAD_BF16)
        B.rad_forward_sample(ctx, L, B.make_sampling(B.RAD_EXACT, 1.0, 1), dev(x, B.RAD_BF16), dev(W, B.RAD_BF16), None,
                             y, st)
        gW = empty((D, N))
        B.rad_backward_dW(ctx, L, st, dev(dy, B.RAD_BF16), gW, None, 0.0)
        want = R.backward_dW(x, dy, np.ones((batch, N), dtype=bool))
        assert rel_err(host(gW), want) < 1e-5          # fp32 sums of exact bf16 products
        B.rad_backward_dW(ctx, L, st, dev(dy, B.RAD_BF16), gW, None, 1.0)
        assert rel_err(host(gW), 2 * want) < 1e-5
    finally:
        B.rad_store_destroy(st)


@pytest.mark.parametrize("relu", [False, True])
@pytest.mark.parametrize("scheme,p", [(3, 0.25), (1, 0.1), (2, 0.25)])
def test_narrow_layer_with_long_contractions(ctx, scheme, p, relu):
    """A narrow bf16 layer with a deep contraction (few output tiles): the forward of a layer without ReLU and
    dW from the store split K over several workgroups per tile and reduce the partial sums afterwards.  All
    three entry points against the oracle on identical inputs, stores compared entry by entry."""
    from paper_2007_10412_amd import binding as B
    from tests.test_gpu_linear import run_layer
    Bt, D, N = 2048, 2304, 200
    rng = np.random.default_rng(400 + scheme)
    x = bf16_data(rng, (Bt, D))
    W = bf16_data(rng, (D, N), 1.0 / np.sqrt(D))
    bias = rng.standard_normal(N).astype(np.float32)
    dy = bf16_data(rng, (Bt, N))
    run_layer(ctx, x, W, bias, dy, scheme, p, seed=11, dtype=B.RAD_BF16, relu=relu)


@pytest.mark.parametrize("N", [256, 1000])
def test_dW_with_segments_longer_than_the_register_budget(ctx, N):
    """The bf16 dW kernel keeps a fixed number of entries per (store row, 256-column bucket) in registers and
    leaves longer segments to a second kernel.  One-bit keys (test hook) make every row keep the lowest columns
    whose key is 0, about half of the first bucket, far more than the kernel holds.  dW is compared with the
    product formed from the store the GPU itself exports, so the check does not depend on the draw."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty, rel_err, TOL
    Bt, D, p = 256, 1024, 0.1
    rng = np.random.default_rng(500 + N)
    x = bf16_data(rng, (Bt, D))
    dy = bf16_data(rng, (Bt, N))
    L = B.make_layer(Bt, D, N, dtype=B.RAD_BF16, relu=False)
    st = B.rad_store_create(ctx, L, B.RAD_FIXEDK_PER_EXAMPLE, p)
    B.rad_debug_key_shift(ctx, 31)
    try:
        B.rad_sample_pack(ctx, B.make_sampling(B.RAD_FIXEDK_PER_EXAMPLE, p, 3), dev(x, B.RAD_BF16), st)
        rp, col, val = B.rad_store_export_csr(ctx, st, Bt)
        seg0 = np.array([np.count_nonzero(col[rp[b]:rp[b + 1]] < 256) for b in range(Bt)])
        assert seg0.min() > 60, seg0.min()          # longer than the 56 entries the kernel holds
        gW = empty((D, N))
        B.rad_backward_dW(ctx, L, st, dev(dy, B.RAD_BF16), gW, None, 0.0)
        xt = np.zeros((Bt, D), dtype=np.float64)
        for b in range(Bt):
            xt[b, col[rp[b]:rp[b + 1]]] = val[rp[b]:rp[b + 1]]
        want = R.backward_dW(xt, dy, np.ones((Bt, N), dtype=bool))
        assert rel_err(host(gW), want) < TOL[B.RAD_BF16]
        assert rel_err(host(gW)[:256], want[:256]) < 1e-4        # fp32 sums of exact products
    finally:
        B.rad_debug_key_shift(ctx, 0)
        B.rad_store_destroy(st)


@pytest.mark.parametrize("relu", [False, True])
def test_forward_wide_layer_ragged_width(ctx, relu):
    """A 2048 x 320 x 4040 layer: 128 tile columns' worth of workgroups whose last tile column ends after 200 of
    its 256 columns (whole 16-byte vectors).  The loads of that tile are clamped to the operand and the epilogue
    guards its stores: y element by element, the ReLU bits, and the packed sample of x."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty, unpack_bits, rel_err, assert_bits_match, TOL
    Bt, d_in, N = 2048, 320, 4040
    rng = np.random.default_rng(77)
    x = bf16_data(rng, (Bt, d_in))
    W = bf16_data(rng, (d_in, N), 1.0 / np.sqrt(d_in))
    bias = rng.standard_normal(N).astype(np.float32)
    print("forward B=%d D=%d N=%d relu=%d" % (Bt, d_in, N, relu), flush=True)
    L = B.make_layer(Bt, d_in, N, dtype=B.RAD_BF16, relu=relu, has_bias=True)
    st = B.rad_store_create(ctx, L, B.RAD_FIXEDK_PER_EXAMPLE, 0.25)
    try:
        y = empty((Bt, N), B.RAD_BF16)
        y.fill_(7.0)        # nothing outside the N columns of a row may be written: the buffer is exactly [Bt, N]
        B.rad_forward_sample(ctx, L, B.make_sampling(B.RAD_FIXEDK_PER_EXAMPLE, 0.25, 7), dev(x, B.RAD_BF16),
                             dev(W, B.RAD_BF16), dev(bias), y, st)
        h, oy, _ = R.linear_forward(x, W, bias, relu, B.RAD_BF16)
        assert rel_err(host(y), oy) < TOL[B.RAD_BF16]
        assert np.max(np.abs(host(y) - oy)) <= 2.0 ** -7 * max(1.0, np.max(np.abs(oy)))
        if relu:
            bits = unpack_bits(B.rad_store_export_bits(ctx, st, Bt, N), N)
            assert_bits_match(bits, h, "relu bits")
    finally:
        B.rad_store_destroy(st)


@pytest.mark.parametrize("N,beta", [(2048, 0.0), (2048, 1.0), (2040, 0.0)])
def test_dW_from_a_wide_store_through_the_dense_operand(ctx, N, beta):
    """dW of a 1024 x 4096 x N layer without ReLU from a sampled store (fraction 0.1): wide enough that the store is
    unpacked into a transient dense operand and contracted by the dense kernel (N = 2040: its last tile column is
    ragged; beta = 1: the accumulating form).  Against the oracle on the store the GPU itself packed."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty, assert_grad_close, TOL
    Bt, D = 1024, 4096
    rng = np.random.default_rng(500 + N)
    x = bf16_data(rng, (Bt, D))
    W = bf16_data(rng, (D, N), 1.0 / 64)
    dy = bf16_data(rng, (Bt, N))
    print("dW dense route B=%d D=%d N=%d beta=%g" % (Bt, D, N, beta), flush=True)
    L = B.make_layer(Bt, D, N, dtype=B.RAD_BF16, relu=False)
    st = B.rad_store_create(ctx, L, B.RAD_FIXEDK_PER_EXAMPLE, 0.1)
    try:
        y = empty((Bt, N), B.RAD_BF16)
        B.rad_forward_sample(ctx, L, B.make_sampling(B.RAD_FIXEDK_PER_EXAMPLE, 0.1, 3), dev(x, B.RAD_BF16),
                             dev(W, B.RAD_BF16), None, y, st)
        _, _, _, xt = R.sample_pack(x, B.RAD_FIXEDK_PER_EXAMPLE, 0.1, 3, 0, 0, B.RAD_BF16)
        want = R.backward_dW(xt, dy, np.ones((Bt, N), dtype=bool))
        gW = empty((D, N))
        start = rng.standard_normal((D, N)).astype(np.float32)
        gW.copy_(dev(start))
        B.rad_backward_dW(ctx, L, st, dev(dy, B.RAD_BF16), gW, None, beta)
        assert_grad_close(host(gW), want + beta * start, TOL[B.RAD_BF16], Bt, "dW")
    finally:
        B.rad_store_destroy(st)

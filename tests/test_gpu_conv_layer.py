"""GPU parity of the single-layer entry points on a convolution layer (RAD_CONV2D): rad_forward_sample,
rad_backward_dW, rad_backward_dX against the oracle's convolution, on identical inputs."""
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


def run_conv_layer(ctx, Bt, ci, co, hw, ks, scheme, p, relu, has_bias, seed, index_free=False):
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty, unpack_bits, assert_grad_close, assert_bits_match
    print("conv layer B=%d ci=%d co=%d hw=%d ks=%d scheme=%d p=%g relu=%d bias=%d" % (Bt, ci, co, hw, ks, scheme, p, relu,
                                                                                      has_bias), flush=True)
    rng = np.random.default_rng(seed)
    pad = (ks - 1) // 2
    x = rng.standard_normal((Bt, ci, hw, hw)).astype(np.float32)
    W = (rng.standard_normal((ci, ks, ks, co)) / np.sqrt(ci * ks * ks)).astype(np.float32)
    bias = (0.1 * rng.standard_normal(co)).astype(np.float32) if has_bias else None
    dy = rng.standard_normal((Bt, co, hw, hw)).astype(np.float32)
    d_in, d_out = ci * hw * hw, co * hw * hw
    L = B.make_layer(Bt, d_in, d_out, relu=relu, has_bias=has_bias, conv=(ci, hw, hw, co, ks, ks, pad))
    st = B.rad_store_create(ctx, L, scheme, p)
    try:
        if index_free:
            B.rad_store_set_index_free(ctx, st, True)
        sm = B.make_sampling(scheme, p, seed, 3, 0)
        gx, gWt = dev(x), dev(W)
        y = empty((Bt, co, hw, hw))
        B.rad_forward_sample(ctx, L, sm, gx, gWt, None if bias is None else dev(bias), y, st)
        # the flattened input is what is sampled (Figure 5)
        rp, col, val = B.rad_store_export_csr(ctx, st, Bt)
        orp, ocol, oval, xt = R.sample_pack(x.reshape(Bt, d_in), scheme, p, seed, 3, 0)
        assert np.array_equal(rp, orp) and np.array_equal(col, ocol)
        assert np.array_equal(val.view(np.uint32), oval.view(np.uint32))
        h, oy, obits = R.conv2d_forward(x, W, bias, pad, relu)
        K = ci * ks * ks
        assert_grad_close(host(y), oy, 1e-4, K, "y")
        if relu:
            bits = unpack_bits(B.rad_store_export_bits(ctx, st, Bt, d_out), d_out)
            assert_bits_match(bits, h.reshape(Bt, d_out), "relu bits")
            bits = bits.reshape(Bt, co, hw, hw)
        else:
            bits = np.ones((Bt, co, hw, hw), dtype=bool)
        g = dy.astype(np.float64) * bits
        gdy = dev(dy)
        gW, gdb = empty((ci, ks, ks, co)), (empty((co,)) if has_bias else None)
        B.rad_backward_dW(ctx, L, st, gdy, gW, gdb, 0.0)
        Kw = Bt * hw * hw
        assert_grad_close(host(gW).reshape(K, co), R.conv2d_dW(xt.reshape(x.shape), g, ks, ks, pad).reshape(K, co), 1e-4,
                          Kw, "dW", c=32.0)
        if has_bias:
            assert_grad_close(host(gdb), g.sum(axis=(0, 2, 3)), 1e-4, Kw, "db", c=32.0)
        gdX = empty((Bt, ci, hw, hw))
        B.rad_backward_dX(ctx, L, st, gdy, gWt, gdX)
        assert_grad_close(host(gdX).reshape(Bt, d_in), R.conv2d_dX(g, W, pad, (hw, hw)).reshape(Bt, d_in), 1e-4, co * ks * ks,
                          "dX")
        with pytest.raises(B.RadError) as e:
            B.rad_backward_dW(ctx, L, st, gdy, gW, gdb, 1.0)
        assert e.value.status == B.RAD_ERR_UNSUPPORTED
    finally:
        B.rad_store_destroy(st)


@pytest.mark.parametrize("scheme,p", [(1, 0.1), (3, 0.25), (2, 0.25), (0, 1.0), (5, 0.25)])
def test_conv_layer_3x3(ctx, scheme, p):
    run_conv_layer(ctx, 6, 8, 12, 16, 3, scheme, p, relu=True, has_bias=True, seed=scheme + 1)


def test_conv_layer_config3_shapes(ctx):
    """The three convolutions of the small CNN (3 -> 16 -> 32 at 32 x 32, 32 -> 64 at 16 x 16), a few examples each."""
    for ci, co, hw in ((3, 16, 32), (16, 32, 32), (32, 64, 16)):
        run_conv_layer(ctx, 5, ci, co, hw, 3, 1, 0.1, relu=True, has_bias=True, seed=ci)


def test_conv_layer_5x5_no_relu_no_bias_index_free(ctx):
    run_conv_layer(ctx, 4, 3, 16, 16, 5, 3, 0.1, relu=False, has_bias=False, seed=9)
    run_conv_layer(ctx, 4, 16, 32, 16, 5, 1, 0.3, relu=True, has_bias=True, seed=10, index_free=True)


def test_conv_layer_limits_are_status_codes(ctx):
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, empty
    L = B.make_layer(2, 3 * 10 * 10, 8 * 10 * 10, relu=True, conv=(3, 10, 10, 8, 3, 3, 1))     # 100 positions: not a multiple of 64
    st = B.rad_store_create(ctx, L, 1, 0.5)
    try:
        with pytest.raises(B.RadError) as e:
            B.rad_forward_sample(ctx, L, B.make_sampling(1, 0.5, 1), dev(np.zeros((2, 300), np.float32)),
                                 dev(np.zeros((27, 8), np.float32)), None, empty((2, 800)), st)
        assert e.value.status == B.RAD_ERR_UNSUPPORTED
    finally:
        B.rad_store_destroy(st)

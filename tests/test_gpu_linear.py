"""GPU parity of the single-layer entry points (config 1 and edge shapes):
rad_forward_sample, rad_backward_dW, rad_backward_dX against the oracle."""
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


def run_layer(ctx, x, W, bias, dy, scheme, p, seed, dtype, relu=True, stream_id=0, step=0):
    """Runs the three entry points on the GPU and checks each against the oracle on identical inputs."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import (dev, host, empty, unpack_bits, rel_err, assert_bits_match, assert_grad_close, TOL,
                                U_BF16)
    Bt, D = x.shape
    N = W.shape[1]
    print("layer B=%d D=%d N=%d scheme=%d p=%g dtype=%d relu=%d" % (Bt, D, N, scheme, p, dtype, relu), flush=True)
    L = B.make_layer(Bt, D, N, dtype=dtype, relu=relu, has_bias=bias is not None)
    st = B.rad_store_create(ctx, L, scheme, p)
    try:
        sm = B.make_sampling(scheme, p, seed, stream_id, step)
        dx_, dW_, dbias_ = dev(x, dtype), dev(W, dtype), None if bias is None else dev(bias)
        y = empty((Bt, N), dtype)
        B.rad_forward_sample(ctx, L, sm, dx_, dW_, dbias_, y, st)
        rp, col, val = B.rad_store_export_csr(ctx, st, Bt)
        orp, ocol, oval, xt = R.sample_pack(x, scheme, p, seed, stream_id, step, dtype)
        assert np.array_equal(rp, orp) and np.array_equal(col, ocol)
        assert np.array_equal(val.view(np.uint32), oval.view(np.uint32))
        h, oy, obits = R.linear_forward(x, W, bias, relu, dtype)
        yh = host(y)
        tol = TOL[dtype]
        # identical inputs on both sides: what differs is the fp32 accumulation and, for bf16, one rounding of the output
        out_u = 4 * U_BF16 if dtype == B.RAD_BF16 else 0.0     # one bf16 ulp: a sum at a rounding boundary
        ratios = {"y": assert_grad_close(yh, oy, tol, D, "y", out_u=out_u)[1]}
        if relu:
            bits = unpack_bits(B.rad_store_export_bits(ctx, st, Bt, N), N)
            flips = assert_bits_match(bits, h, "relu bits")
        else:
            bits, flips = np.ones((Bt, N), dtype=bool), 0
        # backward: the oracle gets the GPU's own store and bits (per-kernel parity on identical inputs)
        gdy = dev(dy, dtype)
        gW = empty((D, N))
        gdb = empty((N,)) if bias is not None else None
        B.rad_backward_dW(ctx, L, st, gdy, gW, gdb, 0.0)
        want_dW = R.backward_dW(xt, dy, bits)
        ratios["dW"] = assert_grad_close(host(gW), want_dW, tol, Bt, "dW")[1]
        if bias is not None:
            ratios["db"] = assert_grad_close(host(gdb), R.backward_db(dy, bits), tol, Bt, "db")[1]
        gdX = empty((Bt, D), dtype)
        B.rad_backward_dX(ctx, L, st, gdy, dW_, gdX)
        ratios["dX"] = assert_grad_close(host(gdX), R.backward_dX(dy, bits, W), tol, N, "dX", out_u=out_u)[1]
        # accumulate (beta = 1) doubles the gradient
        B.rad_backward_dW(ctx, L, st, gdy, gW, gdb, 1.0)
        assert_grad_close(host(gW), 2 * want_dW, tol, Bt, "dW beta=1")
        print("  max element error / max|want|: " + " ".join("%s %.1e" % kv for kv in ratios.items()), flush=True)
        return dict(dW=host(gW) / 2, dX=host(gdX), flips=flips, keep=xt != 0)
    finally:
        B.rad_store_destroy(st)


@pytest.mark.parametrize("scheme,p", [(1, 0.1), (3, 0.1), (2, 0.1), (0, 1.0), (1, 1.0), (3, 1.0), (1, 0.5)])
def test_config1_single_layer(ctx, scheme, p):
    from paper_2007_10412_amd import binding as B, synth
    d = synth.single_layer()
    out = run_layer(ctx, d["x"], d["W"], None, d["dy"], scheme, p, seed=1, dtype=B.RAD_F32)
    if scheme == 2:      # "same sample": rows of dW outside the index set stay exactly zero
        m = R.keep_mask(2, p, 1, 0, 0, 1, 784)[0]
        assert np.all(out["dW"][~m] == 0)


def test_dX_does_not_depend_on_the_sample(ctx):
    from paper_2007_10412_amd import binding as B, synth
    d = synth.single_layer()
    a = run_layer(ctx, d["x"], d["W"], None, d["dy"], 1, 0.1, seed=1, dtype=B.RAD_F32)
    b = run_layer(ctx, d["x"], d["W"], None, d["dy"], 3, 0.5, seed=99, dtype=B.RAD_F32)
    assert np.array_equal(a["dX"], b["dX"])


@pytest.mark.parametrize("Bt,D,N", [(1, 5, 3), (7, 37, 10), (150, 300, 10), (130, 260, 70), (64, 1030, 129),
                                    (70, 600, 640), (100, 520, 270)])     # the last two: split-K forward and dX
@pytest.mark.parametrize("scheme", [1, 2, 3])
def test_ragged_shapes_f32(ctx, Bt, D, N, scheme):
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(Bt * 7 + D)
    x = rng.standard_normal((Bt, D)).astype(np.float32)
    W = (rng.standard_normal((D, N)) / np.sqrt(D)).astype(np.float32)
    bias = (0.1 * rng.standard_normal(N)).astype(np.float32)
    dy = rng.standard_normal((Bt, N)).astype(np.float32)
    run_layer(ctx, x, W, bias, dy, scheme, 0.3, seed=5, dtype=B.RAD_F32)


@pytest.mark.parametrize("Bt,D,N", [(128, 576, 576), (128, 1088, 128), (64, 544, 1920), (128, 1600, 64)])
def test_split_k_interior_f32(ctx, Bt, D, N):
    """Whole 64 x 64 tiles and a K that is a multiple of 32 but not of 128: the unguarded split-K kernels run,
    and every split's K range has to be whole 32-deep slices (forward: K = D, dX: K = N)."""
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(Bt + D + N)
    x = rng.standard_normal((Bt, D)).astype(np.float32)
    W = (rng.standard_normal((D, N)) / np.sqrt(D)).astype(np.float32)
    bias = (0.1 * rng.standard_normal(N)).astype(np.float32)
    dy = rng.standard_normal((Bt, N)).astype(np.float32)
    run_layer(ctx, x, W, bias, dy, 1, 0.3, seed=6, dtype=B.RAD_F32)


def test_large_tile_path_f32(ctx):
    """Enough tiles for the 128x128 kernels, ragged in every dimension."""
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(3)
    Bt, D, N = 1800, 1500, 1700
    x = rng.standard_normal((Bt, D)).astype(np.float32)
    W = (rng.standard_normal((D, N)) / np.sqrt(D)).astype(np.float32)
    dy = rng.standard_normal((Bt, N)).astype(np.float32)
    for scheme in (1, 3):
        run_layer(ctx, x, W, None, dy, scheme, 0.1, seed=8, dtype=B.RAD_F32)


@pytest.mark.parametrize("scheme,p", [(3, 0.1), (2, 0.1), (1, 0.1), (3, 0.5), (3, 0.02), (0, 1.0)])
def test_bf16_layer(ctx, scheme, p):
    from paper_2007_10412_amd import binding as B
    from paper_2007_10412_amd.synth import bf16_round
    rng = np.random.default_rng(4)
    Bt, D, N = 512, 1024, 768
    x = bf16_round(rng.standard_normal((Bt, D)))
    W = bf16_round(rng.standard_normal((D, N)) / np.sqrt(D))
    dy = bf16_round(rng.standard_normal((Bt, N)) * 0.01)
    run_layer(ctx, x, W, None, dy, scheme, p, seed=12, dtype=B.RAD_BF16)


def test_bf16_ragged(ctx):
    from paper_2007_10412_amd import binding as B
    from paper_2007_10412_amd.synth import bf16_round
    rng = np.random.default_rng(5)
    Bt, D, N = 200, 520, 1000
    x = bf16_round(rng.standard_normal((Bt, D)))
    W = bf16_round(rng.standard_normal((D, N)) / np.sqrt(D))
    dy = bf16_round(rng.standard_normal((Bt, N)) * 0.01)
    bias = (0.1 * rng.standard_normal(N)).astype(np.float32)
    for scheme in (1, 2, 3):
        run_layer(ctx, x, W, bias, dy, scheme, 0.1, seed=13, dtype=B.RAD_BF16)


def test_unbiased_on_gpu(ctx):
    """Mean of dW over seeds approaches the exact gradient at the closed-form rate (Section 3.2: E[P] = I)."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty
    rng = np.random.default_rng(21)
    Bt, D, N, p, S = 32, 96, 16, 0.25, 400
    x = rng.standard_normal((Bt, D)).astype(np.float32)
    W = (rng.standard_normal((D, N)) / np.sqrt(D)).astype(np.float32)
    dy = rng.standard_normal((Bt, N)).astype(np.float32)
    L = B.make_layer(Bt, D, N)
    h, _, bits = R.linear_forward(x, W, None, True)
    exact = R.backward_dW(x, dy, bits)
    g2 = (dy.astype(np.float64) * bits) ** 2
    for scheme in (1, 3):
        st = B.rad_store_create(ctx, L, scheme, p)
        gx, gWt, gdy, y, gW = dev(x), dev(W), dev(dy), empty((Bt, N)), empty((D, N))
        acc = np.zeros((D, N))
        for s in range(S):
            B.rad_forward_sample(ctx, L, B.make_sampling(scheme, p, s, 0, 0), gx, gWt, None, y, st)
            B.rad_backward_dW(ctx, L, st, gdy, gW, None, 0.0)
            acc += host(gW)
        B.rad_store_destroy(st)
        pi = p if scheme == 1 else R.fixed_k(p, D) / D
        var = (1 / pi - 1) * ((x.astype(np.float64) ** 2).T @ g2).sum()
        err = np.linalg.norm(acc / S - exact)
        assert err < 4 * np.sqrt(var / S) and err > 0.1 * np.sqrt(var / S)


@pytest.mark.parametrize("Bt,D,N", [
    (3072, 320, 2816),     # forward on 256x256 tiles (132 of them), ragged N tail handled by the 11th column
    (3072, 2816, 328),     # dX on 256x256 tiles
    (328, 3072, 2816),     # dW on 256x256 tiles, K (= batch) with a ragged tail
])
def test_bf16_256_tiles(ctx, Bt, D, N):
    """Shapes that reach the one-workgroup-per-CU 256x256 kernels config 4 runs on."""
    from paper_2007_10412_amd import binding as B
    from paper_2007_10412_amd.synth import bf16_round
    rng = np.random.default_rng(Bt + D)
    x = bf16_round(rng.standard_normal((Bt, D)))
    W = bf16_round(rng.standard_normal((D, N)) / np.sqrt(D))
    dy = bf16_round(rng.standard_normal((Bt, N)) * 0.01)
    for scheme, p in ((3, 0.1), (1, 0.5), (3, 0.02), (2, 0.1)):
        run_layer(ctx, x, W, None, dy, scheme, p, seed=31, dtype=B.RAD_BF16)

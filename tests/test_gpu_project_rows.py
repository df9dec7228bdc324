"""GPU parity of the projection with a Rademacher matrix per example (Appendix A, "different project"; Section 3.2,
P = R R^T / k): every sign against the oracle, the stored projections and the gradients within tolerance, over
row counts k on both sides of the 128-sign Philox call and widths that are not multiples of the workgroup."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

from oracle import rad_oracle as R

SCHEME = 7


@pytest.fixture(scope="module")
def ctx():
    from paper_2007_10412_amd import binding as B
    c = B.rad_ctx_create()
    yield c
    B.rad_ctx_destroy(c)


@pytest.mark.parametrize("d,p,dtype", [(96, 0.25, 0), (300, 0.5, 0), (1024, 0.1, 1), (130, 1.0, 1)])
def test_signs_are_the_oracles(ctx, d, p, dtype):
    """Example b projects the unit vector e_(b mod d): its stored row is row b mod d of its own R_b / sqrt(k).
    With 2 d examples every row index is checked under two different matrices."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev
    k = R.fixed_k(p, d)
    rows = 2 * d
    x = np.zeros((rows, d), dtype=np.float32)
    x[np.arange(rows), np.arange(rows) % d] = 1.0
    st = B.rad_store_create(ctx, B.make_layer(rows, d, 8, dtype=dtype, relu=False), SCHEME, p)
    try:
        B.rad_sample_pack(ctx, B.make_sampling(SCHEME, p, 1234567, 3, 1), dev(x, dtype), st)
        rp, col, val = B.rad_store_export_csr(ctx, st, rows)
    finally:
        B.rad_store_destroy(st)
    assert np.array_equal(rp, np.arange(rows + 1) * k) and np.array_equal(col, np.tile(np.arange(k), rows))
    got = val.reshape(rows, k)
    inv = R.to_storage(np.array([np.float64(np.float32(1 / np.sqrt(k)))]), dtype)[0]
    for b in range(rows):
        Rb = R.rademacher_matrix_of_example(p, 1234567, 3, 1, b, d)
        assert np.array_equal(got[b], Rb[b % d] * inv), b


def _layer(ctx, Bt, D, N, p, dtype, seed):
    from paper_2007_10412_amd import binding as B
    from paper_2007_10412_amd.synth import bf16_round
    from tests.gpu_util import dev, host, empty, unpack_bits, rel_err, assert_bits_match, TOL
    rng = np.random.default_rng(Bt + D)
    rnd = bf16_round if dtype == B.RAD_BF16 else (lambda a: np.asarray(a, np.float32))
    x = rnd(rng.standard_normal((Bt, D)))
    W = rnd(rng.standard_normal((D, N)) / np.sqrt(D))
    dy = rnd(rng.standard_normal((Bt, N)) * 0.1)
    print("project per example: layer B=%d D=%d N=%d p=%g dtype=%d" % (Bt, D, N, p, dtype), flush=True)
    L = B.make_layer(Bt, D, N, dtype=dtype, relu=True)
    st = B.rad_store_create(ctx, L, SCHEME, p)
    tol = TOL[dtype]
    try:
        sm = B.make_sampling(SCHEME, p, seed, 2, 0)
        y = empty((Bt, N), dtype)
        B.rad_forward_sample(ctx, L, sm, dev(x, dtype), dev(W, dtype), None, y, st)
        rp, col, val = B.rad_store_export_csr(ctx, st, Bt)
        k = R.fixed_k(p, D)
        z_ref, xt_ref = R.project_store(x, p, seed, 2, 0, dtype, per_example=True)
        z = val.reshape(Bt, k)
        assert rel_err(z, z_ref) < tol
        if dtype == B.RAD_F32:       # fp32 sums of D terms of size |x|: element by element
            assert np.abs(z - z_ref).max() <= 1e-5 * np.abs(z_ref).max()
        stats = B.rad_store_get_stats(ctx, st)
        assert stats["nnz"] == Bt * k and stats["index_bytes"] == 0
        h, oy, _ = R.linear_forward(x, W, None, True, dtype)
        assert rel_err(host(y), oy) < tol
        bits = unpack_bits(B.rad_store_export_bits(ctx, st, Bt, N), N)
        assert_bits_match(bits, h, "relu bits")
        # backward from the GPU's own store and bits: x~_b = z_b R_b^T / sqrt(k)
        inv = np.float64(np.float32(1 / np.sqrt(k)))
        xt = np.stack([(z[b].astype(np.float64) @ R.rademacher_matrix_of_example(p, seed, 2, 0, b, D).T) * inv
                       for b in range(Bt)])
        gW = empty((D, N))
        B.rad_backward_dW(ctx, L, st, dev(dy, dtype), gW, None, 0.0)
        want = R.backward_dW(xt, dy, bits)
        e = rel_err(host(gW), want)
        assert e < tol, ("dW", e)
        B.rad_backward_dW(ctx, L, st, dev(dy, dtype), gW, None, 1.0)
        assert rel_err(host(gW), 2 * want) < tol
        assert rel_err(host(gW) / 2, R.backward_dW(xt_ref, dy, bits)) < 2 * tol
    finally:
        B.rad_store_destroy(st)


@pytest.mark.parametrize("Bt,D,N,p", [(7, 37, 10, 0.3), (150, 784, 300, 0.1), (130, 260, 70, 0.5), (40, 784, 64, 0.25)])
def test_layer_f32(ctx, Bt, D, N, p):
    _layer(ctx, Bt, D, N, p, 0, seed=5)


@pytest.mark.parametrize("Bt,D,N,p", [(256, 1024, 768, 0.1), (260, 520, 136, 0.25), (128, 1024, 256, 0.02)])
def test_layer_bf16(ctx, Bt, D, N, p):
    _layer(ctx, Bt, D, N, p, 1, seed=12)


@pytest.mark.parametrize("dtype,dims,Bt", [(0, (784, 300, 300, 10), 150), (1, (1024, 768, 512, 1000), 256)])
def test_mlp_train_step(ctx, dtype, dims, Bt):
    from paper_2007_10412_amd import binding as B, synth
    from tests.gpu_util import dev, host, empty, rel_err, unpack_bits, TOL
    data = synth.mlp(seed=3, batch=Bt, dims=dims, pixels=(dtype == 0), bf16=(dtype == 1))
    p, seed = 0.1, 6
    m = B.rad_model_create_mlp(ctx, dtype, Bt, list(dims), False, SCHEME, p)
    try:
        params = [dev(w, dtype) for w in data["Ws"]]
        grads = [empty(w.shape) for w in data["Ws"]]
        loss = B.rad_train_step(ctx, m, B.make_sampling(SCHEME, p, seed, 10, 0), dev(data["x"], dtype),
                                dev(data["labels"]), params, grads)
        gbits = []
        for l in range(2):
            st = B.rad_model_store(m, l)
            gbits.append(unpack_bits(B.rad_store_export_bits(ctx, st, Bt, dims[l + 1]), dims[l + 1]))
        ref = R.mlp_train_step(data["x"], data["labels"], data["Ws"], None, SCHEME, p, seed, stream_base=10,
                               dtype=dtype, bits_override=gbits)
        tol = TOL[dtype]
        assert abs(loss - ref["loss"]) < (1e-5 if dtype == 0 else 2e-2) * max(1.0, abs(ref["loss"]))
        for l in range(3):
            rp, col, val = B.rad_store_export_csr(ctx, B.rad_model_store(m, l), Bt)
            assert rel_err(val, ref["stores"][l][2]) < tol, ("z", l)
            e = rel_err(host(grads[l]), ref["dW"][l])
            assert e < 2 * tol, ("dW", l, e)
    finally:
        B.rad_model_destroy(m)


def test_unbiased_over_seeds(ctx):
    """Mean over seeds against the exact gradient, within four standard errors of the closed-form variance
    sum_b g^2 (|x_b|^2 - x_bj^2) / k of independent matrices."""
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty
    rng = np.random.default_rng(8)
    Bt, D, N, p, S = 32, 96, 16, 0.25, 400
    x = rng.standard_normal((Bt, D)).astype(np.float32)
    dy = rng.standard_normal((Bt, N)).astype(np.float32)
    x64, g = x.astype(np.float64), dy.astype(np.float64)
    exact = x64.T @ g
    L = B.make_layer(Bt, D, N, relu=False)
    st = B.rad_store_create(ctx, L, SCHEME, p)
    try:
        gx, gdy, gW = dev(x), dev(dy), empty((D, N))
        acc = np.zeros_like(exact); acc2 = np.zeros_like(exact)
        for s in range(S):
            B.rad_sample_pack(ctx, B.make_sampling(SCHEME, p, s, 0, 0), gx, st)
            B.rad_backward_dW(ctx, L, st, gdy, gW, None, 0.0)
            e = host(gW).astype(np.float64)
            acc += e; acc2 += e * e
    finally:
        B.rad_store_destroy(st)
    k = R.fixed_k(p, D)
    var_cf = (((x64**2).sum(axis=1, keepdims=True) - x64**2).T @ g**2) / k
    err = np.linalg.norm(acc / S - exact)
    assert 0 < err < 4 * np.sqrt(var_cf.sum() / S)
    var = acc2 / S - (acc / S) ** 2
    assert abs(var.sum() / var_cf.sum() - 1) < 0.15


def test_unsupported_uses_are_status_codes(ctx):
    from paper_2007_10412_amd import binding as B
    with pytest.raises(B.RadError) as e:
        B.rad_model_create_cnn(ctx, 4, [3, 8], [0], 3, 8, 8, 10, SCHEME, 0.5)      # linear layers and MLP / RNN models only
    assert e.value.status == B.RAD_ERR_UNSUPPORTED
    with pytest.raises(B.RadError) as e:
        B.rad_store_create(ctx, B.make_layer(8, 65000, 8, relu=False), SCHEME, 0.9)     # k above the limit
    assert e.value.status == B.RAD_ERR_UNSUPPORTED

"""Index-free storage: the store keeps values only and the backward pass draws the columns again.  Everything
must come out exactly as with stored columns (same kernels, same data), at the paper's stored size."""
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


@pytest.mark.parametrize("dtype", [0, 1])
@pytest.mark.parametrize("scheme,p", [(1, 0.1), (3, 0.1), (5, 0.1), (3, 0.5), (4, 0.25)])
def test_layer_equals_indexed_store(ctx, scheme, p, dtype):
    from paper_2007_10412_amd import binding as B
    from paper_2007_10412_amd.synth import bf16_round
    from tests.gpu_util import dev, host, empty
    rng = np.random.default_rng(scheme * 10 + dtype)
    Bt, D, N = (300, 1000, 200) if dtype == 0 else (512, 1024, 768)
    rnd = bf16_round if dtype == 1 else (lambda a: np.asarray(a, np.float32))
    x = rnd(rng.standard_normal((Bt, D)))
    W = rnd(rng.standard_normal((D, N)) / np.sqrt(D))
    dy = rnd(rng.standard_normal((Bt, N)) * 0.1)
    L = B.make_layer(Bt, D, N, dtype=dtype, relu=True)
    out = {}
    for mode in (False, True):
        st = B.rad_store_create(ctx, L, scheme, p)
        try:
            if mode:
                B.rad_store_set_index_free(ctx, st, True)
            y = empty((Bt, N), dtype)
            B.rad_forward_sample(ctx, L, B.make_sampling(scheme, p, 21, 1, 0), dev(x, dtype), dev(W, dtype), None, y, st)
            gW = empty((D, N))
            B.rad_backward_dW(ctx, L, st, dev(dy, dtype), gW, None, 0.0)
            out[mode] = dict(csr=B.rad_store_export_csr(ctx, st, Bt), dW=host(gW), stats=B.rad_store_get_stats(ctx, st))
        finally:
            B.rad_store_destroy(st)
    for a, b in zip(out[False]["csr"], out[True]["csr"]):
        assert np.array_equal(a, b)
    assert np.array_equal(out[False]["dW"], out[True]["dW"])
    nnz = out[True]["stats"]["nnz"]
    assert out[True]["stats"]["value_bytes"] == out[False]["stats"]["value_bytes"]
    assert out[False]["stats"]["index_bytes"] - out[True]["stats"]["index_bytes"] == 2 * nnz
    # and against the oracle
    orp, ocol, oval, _ = R.sample_pack(x, scheme, p, 21, 1, 0, dtype)
    assert np.array_equal(out[True]["csr"][0], orp) and np.array_equal(out[True]["csr"][1], ocol)
    assert np.array_equal(out[True]["csr"][2].view(np.uint32), oval.view(np.uint32))


@pytest.mark.parametrize("dtype,dims,Bt,scheme", [(0, (784, 300, 300, 10), 150, 3), (1, (1024, 768, 512, 1000), 512, 3),
                                                  (1, (1024, 768, 512, 1000), 512, 1)])
def test_mlp_step_equals_indexed_model(ctx, dtype, dims, Bt, scheme):
    from paper_2007_10412_amd import binding as B, synth
    from tests.gpu_util import dev, host, empty
    data = synth.mlp(seed=3, batch=Bt, dims=dims, pixels=(dtype == 0), bf16=(dtype == 1))
    p = 0.1
    res = {}
    for mode in (False, True):
        m = B.rad_model_create_mlp(ctx, dtype, Bt, list(dims), False, scheme, p)
        try:
            if mode:
                B.rad_model_set_index_free(ctx, m, True)
            params = [dev(w, dtype) for w in data["Ws"]]
            grads = [empty(w.shape) for w in data["Ws"]]
            x, labels = dev(data["x"], dtype), dev(data["labels"])
            for seed in (5, 6):          # two steps: the workspace rebuilds are per step
                loss = B.rad_train_step(ctx, m, B.make_sampling(scheme, p, seed, 10, 0), x, labels, params, grads)
            stats = [B.rad_store_get_stats(ctx, B.rad_model_store(m, l)) for l in range(3)]
            res[mode] = dict(loss=loss, grads=[host(g) for g in grads], stats=stats)
        finally:
            B.rad_model_destroy(m)
    assert res[False]["loss"] == res[True]["loss"]
    for a, b in zip(res[False]["grads"], res[True]["grads"]):
        assert np.array_equal(a, b)
    for sa, sb in zip(res[False]["stats"], res[True]["stats"]):
        assert sb["index_bytes"] == sa["index_bytes"] - 2 * sa["nnz"] and sb["value_bytes"] == sa["value_bytes"]


def test_unsupported_uses_are_status_codes(ctx):
    from paper_2007_10412_amd import binding as B
    st = B.rad_store_create(ctx, B.make_layer(8, 64, 8, relu=False), 2, 0.5)
    try:
        with pytest.raises(B.RadError) as e:
            B.rad_store_set_index_free(ctx, st, True)
        assert e.value.status == B.RAD_ERR_UNSUPPORTED
    finally:
        B.rad_store_destroy(st)
    m = B.rad_model_create_rnn(ctx, 8, 4, 1, 32, 10, 1, 0.5)
    try:
        with pytest.raises(B.RadError) as e:
            B.rad_model_set_index_free(ctx, m, True)
        assert e.value.status == B.RAD_ERR_UNSUPPORTED
    finally:
        B.rad_model_destroy(m)
    st = B.rad_store_create(ctx, B.make_layer(8, 64, 8, relu=False), 3, 0.5)
    try:
        B.rad_store_set_index_free(ctx, st, True)
        from tests.gpu_util import dev, empty
        with pytest.raises(B.RadError) as e:          # nothing sampled yet
            B.rad_backward_dW(ctx, B.make_layer(8, 64, 8, relu=False), st, dev(np.zeros((8, 8), np.float32)),
                              empty((64, 8)), None, 0.0)
        assert e.value.status == B.RAD_ERR_PARAM
    finally:
        B.rad_store_destroy(st)

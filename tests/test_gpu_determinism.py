"""Run-to-run determinism: the same seed twice gives bit-identical stores and bit-identical gradients.
Every split-K reduction adds its partial sums in a fixed order (no floating-point atomics on any path these
tests reach), so the gradients are compared exactly, not to a tolerance."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    from paper_2007_10412_amd import binding as B
    c = B.rad_ctx_create()
    yield c
    B.rad_ctx_destroy(c)


def _mlp_twice(ctx, dims, Bt, scheme, p, dtype, seed):
    import torch
    from paper_2007_10412_amd import binding as B, synth
    from tests.gpu_util import dev, host, empty
    data = synth.mlp(seed=17, batch=Bt, dims=dims, pixels=False, bf16=dtype == B.RAD_BF16)
    m = B.rad_model_create_mlp(ctx, dtype, Bt, list(dims), False, scheme, p)
    try:
        params = [dev(w, dtype) for w in data["Ws"]]
        grads = [empty(w.shape) for w in data["Ws"]]
        x, labels = dev(data["x"], dtype), dev(data["labels"])
        runs = []
        for rep in range(2):
            for g in grads:
                g.fill_(float("nan"))
            torch.cuda.synchronize()
            loss = B.rad_train_step(ctx, m, B.make_sampling(scheme, p, seed, 3, 0), x, labels, params, grads)
            stores = [B.rad_store_export_csr(ctx, B.rad_model_store(m, l), Bt) for l in range(len(dims) - 1)]
            runs.append((loss, [host(g).copy() for g in grads], stores))
            if rep == 0:      # another draw in between, so that nothing of the first run is simply left in place
                B.rad_train_step(ctx, m, B.make_sampling(scheme, p, seed + 1, 3, 0), x, labels, params, grads)
        (l0, g0, s0), (l1, g1, s1) = runs
        assert l0 == l1
        for a, b in zip(s0, s1):
            for u, v in zip(a, b):
                assert np.array_equal(u.view(np.uint32) if u.dtype == np.float32 else u,
                                      v.view(np.uint32) if v.dtype == np.float32 else v)
        for l, (a, b) in enumerate(zip(g0, g1)):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), "dW of layer %d differs between two runs" % l
    finally:
        B.rad_model_destroy(m)


# shared scheme at small k: the compact dW splits the batch (K) over several workgroups per tile
@pytest.mark.parametrize("scheme,p", [(1, 0.1), (2, 0.1), (2, 0.02), (3, 0.1), (3, 0.5), (4, 0.1), (5, 0.1), (6, 0.1)])
def test_mlp_bf16_two_runs_identical(ctx, scheme, p):
    from paper_2007_10412_amd import binding as B
    _mlp_twice(ctx, (1024, 2048, 1024, 1000), 2048, scheme, p, B.RAD_BF16, seed=9)


@pytest.mark.parametrize("scheme,p", [(1, 0.1), (2, 0.1), (3, 0.1)])
def test_mlp_f32_two_runs_identical(ctx, scheme, p):
    from paper_2007_10412_amd import binding as B
    _mlp_twice(ctx, (784, 300, 300, 10), 150, scheme, p, B.RAD_F32, seed=4)


@pytest.mark.parametrize("scheme,p", [(1, 0.1), (2, 0.25), (3, 0.25)])
def test_rnn_two_runs_identical(ctx, scheme, p):
    """The recurrent gradients are accumulated chunk by chunk on a second stream, in stream order."""
    from paper_2007_10412_amd import binding as B, synth
    from tests.gpu_util import dev, host, empty
    d = synth.rnn(seed=2, batch=32, T=21, d_input=1, hidden=128, classes=10, identity=True)
    Bt, T, I = d["x"].shape
    m = B.rad_model_create_rnn(ctx, Bt, T, I, 128, 10, scheme, p)
    try:
        names = ["W_ih", "W_hh", "b", "W_ho", "b_o"]
        params = [dev(d[n]) for n in names]
        grads = [empty(d[n].shape) for n in names]
        x, labels = dev(d["x"]), dev(d["labels"])
        out = []
        for rep in range(2):
            B.rad_train_step(ctx, m, B.make_sampling(scheme, p, 31, 0, 0), x, labels, params, grads)
            out.append(([host(g).copy() for g in grads],
                        B.rad_store_export_csr(ctx, B.rad_model_store(m, 0), (T - 1) * Bt)))
        for a, b in zip(out[0][0], out[1][0]):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
        for a, b in zip(out[0][1], out[1][1]):
            assert np.array_equal(a.view(np.uint32) if a.dtype == np.float32 else a,
                                  b.view(np.uint32) if b.dtype == np.float32 else b)
    finally:
        B.rad_model_destroy(m)


def test_cnn_two_runs_identical(ctx):
    from paper_2007_10412_amd import binding as B, synth
    from tests.gpu_util import dev, host, empty
    ch, pool = (3, 8, 12, 16), (0, 1, 1)
    d = synth.cnn(seed=7, batch=10, channels=ch, pool=pool, ksize=3, hw=16, classes=10)
    m = B.rad_model_create_cnn(ctx, 10, list(ch), list(pool), 3, 16, 16, 10, 1, 0.1)
    try:
        params, grads = [], []
        for cv in d["convs"]:
            params += [dev(cv["W"]), dev(cv["b"])]
            grads += [empty(cv["W"].shape), empty(cv["b"].shape)]
        params += [dev(d["fc"][0]), dev(d["fc"][1])]
        grads += [empty(d["fc"][0].shape), empty(d["fc"][1].shape)]
        x, labels = dev(d["x"]), dev(d["labels"])
        out = []
        for rep in range(2):
            B.rad_train_step(ctx, m, B.make_sampling(1, 0.1, 5, 0, 0), x, labels, params, grads)
            out.append([host(g).copy() for g in grads])
        for a, b in zip(out[0], out[1]):
            assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    finally:
        B.rad_model_destroy(m)

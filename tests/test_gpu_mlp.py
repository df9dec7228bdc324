"""GPU parity of rad_train_step on the MLP configurations (2 and 4)."""
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


def run_mlp(ctx, data, dims, scheme, p, seed, dtype, has_bias):
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import (dev, host, empty, unpack_bits, rel_err, assert_bits_match, assert_grad_close, TOL,
                                U_F32, U_BF16)
    Bt = data["x"].shape[0]
    L = len(dims) - 1
    print("mlp B=%d dims=%s scheme=%d p=%g dtype=%d" % (Bt, dims, scheme, p, dtype), flush=True)
    m = B.rad_model_create_mlp(ctx, dtype, Bt, list(dims), has_bias, scheme, p)
    try:
        params, grads = [], []
        for l in range(L):
            params.append(dev(data["Ws"][l], dtype)); grads.append(empty(data["Ws"][l].shape))
            if has_bias:
                params.append(dev(data["bs"][l])); grads.append(empty(data["bs"][l].shape))
        x, labels = dev(data["x"], dtype), dev(data["labels"])
        loss = B.rad_train_step(ctx, m, B.make_sampling(scheme, p, seed, 10, 0), x, labels, params, grads)
        tol = TOL[dtype]
        bs = data["bs"] if has_bias else None
        ref = R.mlp_train_step(data["x"], data["labels"], data["Ws"], bs, scheme, p, seed, stream_base=10, dtype=dtype)
        # sampling decisions never depend on data: masks and indices bit-exact at every layer
        flips, gbits = 0, []
        for l in range(L):
            st = B.rad_model_store(m, l)
            rp, col, val = B.rad_store_export_csr(ctx, st, Bt)
            assert np.array_equal(rp, ref["stores"][l][0]), l
            assert np.array_equal(col, ref["stores"][l][1]), l
            assert rel_err(val, ref["stores"][l][2]) < tol, l
            if l == 0:
                assert np.array_equal(val, ref["stores"][0][2])
            if l < L - 1:
                hb = unpack_bits(B.rad_store_export_bits(ctx, st, Bt, dims[l + 1]), dims[l + 1])
                h = np.asarray(ref["acts"][l], np.float64) @ np.asarray(data["Ws"][l], np.float64)
                if bs is not None:
                    h = h + bs[l][None, :]
                # fp32: a flip needs |h| within accumulation rounding of zero.  bf16: the layer input is the
                # rounded output of the layer below, which the two sides may round to neighbouring bf16 values, so
                # h differs by a few 2^-9 |a W| terms: flips stay within 2e-3 rms(h) of zero, and below 1 % of entries
                flips += assert_bits_match(hb, h, "layer %d" % l, near=1e-5 if dtype == B.RAD_F32 else 2e-3)
                gbits.append(hb)
        assert abs(loss - ref["loss"]) < (1e-5 if dtype == B.RAD_F32 else 2e-2) * max(1.0, abs(ref["loss"]))
        if flips:   # rerun the oracle backward with the GPU's ReLU bits
            ref = R.mlp_train_step(data["x"], data["labels"], data["Ws"], bs, scheme, p, seed, stream_base=10,
                                   dtype=dtype, bits_override=gbits)
        per = 2 if has_bias else 1
        # a whole step: rounded intermediates (layer outputs, dX) feed every gradient, so the element-wise bound
        # takes the unit roundoff of the storage type
        u, cc = (U_F32, 32.0) if dtype == B.RAD_F32 else (U_BF16, 0.25)     # observed at most 4e-3 of max|dW| at full size
        ratios = []
        for l in range(L):
            ratios.append(assert_grad_close(host(grads[l * per]), ref["dW"][l], tol, Bt, "dW %d" % l, acc_u=u, c=cc)[1])
            if has_bias:
                assert_grad_close(host(grads[l * per + 1]), ref["db"][l], tol, Bt, "db %d" % l, acc_u=u, c=cc)
        print("  flips %d; dW max element error / max|want|: %s" % (flips, " ".join("%.1e" % r for r in ratios)), flush=True)
        return dict(loss=loss, grads=[host(g) for g in grads], flips=flips)
    finally:
        B.rad_model_destroy(m)


@pytest.mark.parametrize("scheme,p", [(3, 0.1), (2, 0.1), (1, 0.1), (0, 1.0), (3, 1.0)])
def test_config2_mlp(ctx, scheme, p):
    from paper_2007_10412_amd import binding as B, synth
    data = synth.mlp(seed=1234, batch=150, dims=(784, 300, 300, 10), bias_scale=0.0)
    run_mlp(ctx, data, (784, 300, 300, 10), scheme, p, seed=42, dtype=B.RAD_F32, has_bias=True)


def test_mlp_nonzero_bias_ragged(ctx):
    from paper_2007_10412_amd import binding as B, synth
    data = synth.mlp(seed=5, batch=77, dims=(130, 90, 50, 7), bias_scale=0.1, pixels=False)
    for scheme in (1, 2, 3):
        run_mlp(ctx, data, (130, 90, 50, 7), scheme, 0.3, seed=4, dtype=B.RAD_F32, has_bias=True)


def test_fraction_one_equals_exact_scheme(ctx):
    from paper_2007_10412_amd import binding as B, synth
    data = synth.mlp(seed=9, batch=64, dims=(96, 80, 10))
    a = run_mlp(ctx, data, (96, 80, 10), 0, 1.0, seed=1, dtype=B.RAD_F32, has_bias=False)
    b = run_mlp(ctx, data, (96, 80, 10), 3, 1.0, seed=2, dtype=B.RAD_F32, has_bias=False)
    for ga, gb in zip(a["grads"], b["grads"]):
        np.testing.assert_allclose(ga, gb, rtol=1e-5, atol=1e-7)


@pytest.mark.parametrize("scheme,p", [(3, 0.1), (2, 0.1), (3, 0.5), (2, 0.02)])
def test_bf16_mlp_reduced(ctx, scheme, p):
    """Config 4's structure at a size the oracle finishes in seconds."""
    from paper_2007_10412_amd import binding as B, synth
    dims = (1024, 768, 512, 1000)
    data = synth.mlp(seed=3, batch=512, dims=dims, pixels=False, bf16=True)
    run_mlp(ctx, data, dims, scheme, p, seed=6, dtype=B.RAD_BF16, has_bias=False)


@pytest.mark.parametrize("scheme", [1, 3])
def test_enqueue_only_steps_match_waited_steps(ctx, scheme):
    """loss_host = null only enqueues the step: same stores and gradients as the waited step, no loss."""
    import torch
    from paper_2007_10412_amd import binding as B, synth
    from tests.gpu_util import dev, host, empty
    dims, Bt, p = (512, 384, 256, 100), 256, 0.1
    data = synth.mlp(seed=11, batch=Bt, dims=dims, pixels=False, bf16=True)
    m = B.rad_model_create_mlp(ctx, B.RAD_BF16, Bt, list(dims), False, scheme, p)
    try:
        params = [dev(w, B.RAD_BF16) for w in data["Ws"]]
        grads = [empty(w.shape) for w in data["Ws"]]
        x, labels = dev(data["x"], B.RAD_BF16), dev(data["labels"])
        loss = B.rad_train_step(ctx, m, B.make_sampling(scheme, p, 77, 0, 0), x, labels, params, grads)
        assert np.isfinite(loss)
        want = [host(g).copy() for g in grads]
        csr = [B.rad_store_export_csr(ctx, B.rad_model_store(m, l), Bt) for l in range(3)]
        for seed in (5, 6, 77):     # the last one repeats the waited step's draw
            for g in grads:
                g.fill_(float("nan"))
            torch.cuda.synchronize()   # the fills run on torch's stream, the step on the library's
            assert B.rad_train_step(ctx, m, B.make_sampling(scheme, p, seed, 0, 0), x, labels, params, grads,
                                    want_loss=False) is None
        B.rad_ctx_synchronize(ctx)
        for g, w in zip(grads, want):
            np.testing.assert_array_equal(host(g), w)
        for l in range(3):
            got = B.rad_store_export_csr(ctx, B.rad_model_store(m, l), Bt)
            for a, b in zip(got, csr[l]):
                np.testing.assert_array_equal(a, b)
    finally:
        B.rad_model_destroy(m)

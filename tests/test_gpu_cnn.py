"""GPU parity of rad_train_step on the small CNN (config 3): conv as implicit
im2col GEMM, ReLU bits, 2x2 max pool with 2-bit positions, dW from the sampled
conv inputs, exact transposed-conv dX."""
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


def run_cnn(ctx, d, channels, pool, ksize, hw, classes, scheme, p, seed):
    from paper_2007_10412_amd import binding as B
    from tests.gpu_util import dev, host, empty, rel_err, unpack_bits, assert_grad_close, U_F32
    Bt = d["x"].shape[0]
    nc = len(channels) - 1
    print("cnn B=%d channels=%s pool=%s hw=%d scheme=%d p=%g" % (Bt, channels, pool, hw, scheme, p), flush=True)
    m = B.rad_model_create_cnn(ctx, Bt, list(channels), list(pool), ksize, hw, hw, classes, scheme, p)
    try:
        params, grads = [], []
        for cv in d["convs"]:
            params += [dev(cv["W"]), dev(cv["b"])]
            grads += [empty(cv["W"].shape), empty(cv["b"].shape)]
        params += [dev(d["fc"][0]), dev(d["fc"][1])]
        grads += [empty(d["fc"][0].shape), empty(d["fc"][1].shape)]
        loss = B.rad_train_step(ctx, m, B.make_sampling(scheme, p, seed, 30, 0), dev(d["x"]), dev(d["labels"]),
                                params, grads)
        # near-tie decisions (ReLU sign of a pre-activation within rounding of 0, the larger of two almost
        # equal pooled values) are taken from the GPU and fed to the oracle's backward
        gbits, gargs, size = [], [], hw
        for l in range(nc):
            co = channels[l + 1]
            n = co * size * size
            bits = unpack_bits(B.rad_store_export_bits(ctx, B.rad_model_store(m, l), Bt, n), n)
            gbits.append(bits.reshape(Bt, co, size, size))
            if pool[l]:
                size //= 2
            if pool[l] == 1:
                gargs.append(B.rad_model_export_pool_arg(ctx, m, l, Bt * co * size * size).reshape(Bt, co, size, size))
            else:
                gargs.append(None)
        ref0 = R.cnn_train_step(d["x"], d["labels"], d["convs"], d["fc"], scheme, p, seed, stream_base=30)
        flips = sum(int((gb != t[1]).sum()) for gb, t in zip(gbits, ref0["tape"]))
        swaps = sum(int((ga != t[2]).sum()) for ga, t in zip(gargs, ref0["tape"]) if ga is not None)
        n_bits = sum(gb.size for gb in gbits)
        assert flips <= 1e-4 * n_bits and swaps <= 1e-4 * n_bits, (flips, swaps)
        ref = R.cnn_train_step(d["x"], d["labels"], d["convs"], d["fc"], scheme, p, seed, stream_base=30,
                               bits_override=gbits, arg_override=gargs) if (flips or swaps) else ref0
        assert abs(loss - ref["loss"]) < 1e-5 * max(1.0, abs(ref["loss"])), (loss, ref["loss"])
        for l in range(nc + 1):      # sampling decisions: bit-exact
            rp, col, val = B.rad_store_export_csr(ctx, B.rad_model_store(m, l), Bt)
            assert np.array_equal(rp, ref["stores"][l][0]) and np.array_equal(col, ref["stores"][l][1]), l
            assert rel_err(val, ref["stores"][l][2]) < 1e-5, l
        size = hw
        for l in range(nc):      # a conv gradient sums over batch x positions
            K = Bt * size * size
            assert_grad_close(host(grads[2 * l]), ref["dW"][l], 1e-4, K, "dW %d" % l, acc_u=U_F32, c=32.0)
            assert_grad_close(host(grads[2 * l + 1]), ref["db"][l], 1e-4, K, "db %d" % l, acc_u=U_F32, c=32.0)
            if pool[l]:
                size //= 2
        assert_grad_close(host(grads[2 * nc]), ref["dW_fc"], 1e-4, Bt, "dW fc", acc_u=U_F32, c=32.0)
        assert_grad_close(host(grads[2 * nc + 1]), ref["db_fc"], 1e-4, Bt, "db fc", acc_u=U_F32, c=32.0)
        return flips, swaps
    finally:
        B.rad_model_destroy(m)


@pytest.mark.parametrize("scheme,p", [(1, 0.1), (1, 0.5), (3, 0.25), (2, 0.25), (0, 1.0), (1, 1.0)])
def test_cnn_small(ctx, scheme, p):
    from paper_2007_10412_amd import synth
    ch, pool = (3, 8, 12, 16), (0, 1, 1)
    d = synth.cnn(seed=7, batch=6, channels=ch, pool=pool, ksize=3, hw=16, classes=10)
    for cv in d["convs"]:
        cv["b"] = (0.05 * np.random.default_rng(1).standard_normal(cv["b"].shape)).astype(np.float32)
    run_cnn(ctx, d, ch, pool, 3, 16, 10, scheme, p, seed=3)


def test_cnn_5x5_kernels(ctx):
    from paper_2007_10412_amd import synth
    ch, pool = (2, 5, 7), (1, 0)
    d = synth.cnn(seed=8, batch=4, channels=ch, pool=pool, ksize=5, hw=16, classes=7)
    run_cnn(ctx, d, ch, pool, 5, 16, 7, 1, 0.3, seed=4)


def test_config3_reduced_batch(ctx):
    """Config 3's network (3->16->32->64 at 32x32, two pools, FC 4096->10) at batch 24: the oracle's
    fp64 einsum convolutions take minutes at 150; every per-example shape is the real one."""
    from paper_2007_10412_amd import synth
    ch, pool = (3, 16, 32, 64), (0, 1, 1)
    d = synth.cnn(seed=1234, batch=24, channels=ch, pool=pool, ksize=3, hw=32, classes=10)
    run_cnn(ctx, d, ch, pool, 3, 32, 10, 1, 0.1, seed=5)


@pytest.mark.parametrize("scheme,p", [(1, 0.1), (3, 0.25), (0, 1.0)])
def test_cnn_paper_architecture_with_average_pools(ctx, scheme, p):
    """The convolutional architecture of Appendix A (5x5 convolutions with 16, 32, 32, 32 feature maps and 2
    zero padding, 2x2 average pools after the second and fourth, linear 2048 -> 10) at batch 6: loss, stores
    and every gradient against the oracle.  The average pool keeps nothing for the backward pass."""
    from paper_2007_10412_amd import synth
    ch, pool = (3, 16, 32, 32, 32), (0, 2, 0, 2)
    d = synth.cnn(seed=9, batch=6, channels=ch, pool=pool, ksize=5, hw=32, classes=10)
    for cv in d["convs"]:
        cv["b"] = (0.05 * np.random.default_rng(3).standard_normal(cv["b"].shape)).astype(np.float32)
    run_cnn(ctx, d, ch, pool, 5, 32, 10, scheme, p, seed=6)


def test_cnn_mixed_pools_and_bad_pool_kind(ctx):
    from paper_2007_10412_amd import binding as B, synth
    for pool in ((2, 1, 0), (1, 2, 0)):
        ch = (3, 8, 8, 16)
        d = synth.cnn(seed=10, batch=4, channels=ch, pool=pool, ksize=3, hw=32, classes=5)
        run_cnn(ctx, d, ch, pool, 3, 32, 5, 1, 0.3, seed=8)
    with pytest.raises(B.RadError):
        B.rad_model_create_cnn(ctx, 4, [3, 8], [3], 3, 16, 16, 5, 1, 0.3)

"""GPU parity of rad_optimizer_step (SGD and Adam with an l2 term, fp32 parameters and bf16 parameters with fp32
master copies) against the oracle's fp64 updates, element by element; and a few whole iterations
(rad_train_step followed by rad_optimizer_step) of a small MLP against the oracle's.

Tolerance.  The kernel evaluates the update in fp32: the moments are sums of two products (relative error of
a few 2^-24 per step), the step lr m^ / (sqrt(v^) + eps) a handful of correctly rounded operations, so the
change of w agrees to about 1e-6 relative and w itself to one more rounding of w per step: the bound used is
2^-20 |w| + 2e-7 per step for steps of size 0.01 to 0.1."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

from oracle import rad_oracle as R


@pytest.fixture(scope="module")
def ctx():
    from paper_2007_10412_amd import binding as B
    c = B.rad_ctx_create()
    yield c
    B.rad_ctx_destroy(c)


def close(got, want, scale, what):
    got = np.asarray(got, np.float64); want = np.asarray(want, np.float64)
    bound = 2.0 ** -20 * np.abs(want) + scale
    bad = np.abs(got - want) > bound
    assert not bad.any(), (what, int(bad.sum()), float(np.abs(got - want).max()))


SIZES = [1, 3, 257, 4096 * 33 + 2, 0, 1024]


@pytest.mark.parametrize("kind", ["sgd", "adam"])
@pytest.mark.parametrize("offset", [0, 1])
def test_fp32_updates(ctx, kind, offset):
    """Tensors of ragged sizes (vector body and scalar tail; offset 1 starts every array one element off a
    16-byte boundary, which takes the scalar kernel throughout), five steps with gradients of mixed magnitude."""
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(7 + offset)
    adam = kind == "adam"
    lr, l2 = (1e-2, 1e-3) if adam else (5e-2, 1e-2)
    opt = B.make_optimizer(B.RAD_ADAM if adam else B.RAD_SGD, lr, l2, 0.9, 0.99, 1e-7)

    def devbuf(a):
        t = torch.zeros(a.size + offset, device="cuda", dtype=torch.float32)
        v = t[offset:]
        v.copy_(torch.from_numpy(a))
        return v
    w_ref = [rng.standard_normal(n) .astype(np.float32).astype(np.float64) for n in SIZES]
    m_ref = [np.zeros(n) for n in SIZES]; v_ref = [np.zeros(n) for n in SIZES]
    w = [devbuf(a.astype(np.float32)) for a in w_ref]
    m = [devbuf(np.zeros(n, np.float32)) for n in SIZES]; v = [devbuf(np.zeros(n, np.float32)) for n in SIZES]
    gmax = [np.zeros(n) for n in SIZES]
    werr = [np.zeros(n) for n in SIZES]
    print("optimiser %s offset %d" % (kind, offset), flush=True)
    for t in range(1, 6):
        gs = [(rng.standard_normal(n) * 10.0 ** rng.integers(-4, 2, n)).astype(np.float32) for n in SIZES]
        g = [devbuf(a) for a in gs]
        B.rad_optimizer_step(ctx, opt, t, B.RAD_F32, w, g, m if adam else None, v if adam else None)
        B.rad_ctx_synchronize(ctx)
        for i, n in enumerate(SIZES):
            if adam:
                w_ref[i], m_ref[i], v_ref[i] = R.adam_step(w_ref[i], gs[i], m_ref[i], v_ref[i], t, lr, 0.9, 0.99, 1e-7, l2)
            else:
                w_ref[i] = R.sgd_step(w_ref[i], gs[i], lr, l2)
            gmax[i] = np.maximum(gmax[i], np.abs(gs[i]) + l2 * np.abs(w_ref[i]))
            # where g + l2 w cancels to the size of eps the step is ill-conditioned: an error dm of the first
            # moment moves w by lr dm / ((sqrt(v^) + eps)(1 - beta1^t)), and dm is a few roundings of the largest term
            werr[i] += 2e-7
            if adam:
                werr[i] += lr * 4e-7 * gmax[i] / ((np.sqrt(v_ref[i] / (1 - 0.99 ** t)) + 1e-7) * (1 - 0.9 ** t))
            close(w[i].cpu().numpy(), w_ref[i], werr[i], (kind, "w", t, n))
            if adam:     # m is a sum with cancellation: its error scales with the largest term, not with m
                close(m[i].cpu().numpy(), m_ref[i], 2e-7 * gmax[i], (kind, "m", t, n))
                close(v[i].cpu().numpy(), v_ref[i], 1e-8 * gmax[i] ** 2, (kind, "v", t, n))   # g + l2 w cancels too


def test_bf16_parameters_follow_their_master_copies(ctx):
    """Config 4's widest tensor (4096 x 4096): the fp32 master copy against the oracle, every element; the bf16
    parameter is the master copy rounded to nearest even, bit for bit."""
    from paper_2007_10412_amd import binding as B
    rng = np.random.default_rng(11)
    n = 4096 * 4096
    w0 = (rng.standard_normal(n) / 64).astype(np.float32)
    master = torch.from_numpy(w0).cuda()
    wb = master.to(torch.bfloat16)
    m = torch.zeros(n, device="cuda"); v = torch.zeros(n, device="cuda")
    opt = B.make_optimizer(B.RAD_ADAM, 1e-3, 1e-4)
    w_ref, m_ref, v_ref = w0.astype(np.float64), np.zeros(n), np.zeros(n)
    for t in (1, 2):
        g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
        B.rad_optimizer_step(ctx, opt, t, B.RAD_BF16, [wb], [torch.from_numpy(g).cuda()], [m], [v], [master])
        B.rad_ctx_synchronize(ctx)
        w_ref, m_ref, v_ref = R.adam_step(w_ref, g, m_ref, v_ref, t, 1e-3, l2=1e-4)
        mg = master.cpu().numpy()
        close(mg, w_ref, 4e-6 * 1e-3 * t, ("master", t))
        want_bits = (R.round_bf16(mg).view(np.uint32) >> 16).astype(np.uint16)
        got_bits = wb.view(torch.int16).cpu().numpy().view(np.uint16)
        assert np.array_equal(got_bits, want_bits), t


def test_argument_checks(ctx):
    from paper_2007_10412_amd import binding as B
    w = torch.zeros(8, device="cuda"); g = torch.zeros(8, device="cuda")
    wb = w.to(torch.bfloat16)
    adam, sgd = B.make_optimizer(B.RAD_ADAM, 1e-3), B.make_optimizer(B.RAD_SGD, 1e-3)
    for bad in (lambda: B.rad_optimizer_step(ctx, adam, 0, B.RAD_F32, [w], [g], [w], [w]),       # step numbers from 1
                lambda: B.rad_optimizer_step(ctx, adam, 1, B.RAD_F32, [w], [g]),                  # no moments
                lambda: B.rad_optimizer_step(ctx, sgd, 1, B.RAD_BF16, [wb], [g]),                 # no master copy
                lambda: B.rad_optimizer_step(ctx, B.make_optimizer(7, 1e-3), 1, B.RAD_F32, [w], [g]),
                lambda: B.rad_optimizer_step(ctx, B.make_optimizer(B.RAD_SGD, -1.0), 1, B.RAD_F32, [w], [g]),
                lambda: B.rad_optimizer_step(ctx, B.make_optimizer(B.RAD_ADAM, 1e-3, beta1=1.0), 1, B.RAD_F32, [w], [g], [w], [w])):
        with pytest.raises(B.RadError):
            bad()
    assert float(w.abs().sum()) == 0.0          # a rejected call launches nothing


def test_training_iterations_match_the_oracle(ctx):
    """Three iterations of the fully connected architecture of Appendix A (784-300-300-300-10, batch 150,
    different samples per example, fraction 0.1) with Adam: step t samples with seed t; losses and weights
    against the oracle running the same iterations."""
    from paper_2007_10412_amd import binding as B, synth
    from tests.gpu_util import dev, host, empty, rel_err
    dims = (784, 300, 300, 300, 10)
    data = synth.mlp(seed=5, batch=150, dims=dims, bias_scale=0.0)
    L = len(dims) - 1
    model = B.rad_model_create_mlp(ctx, B.RAD_F32, 150, list(dims), True, B.RAD_FIXEDK_PER_EXAMPLE, 0.1)
    try:
        params, grads, ms, vs, ref_p = [], [], [], [], []
        for l in range(L):
            for a in (data["Ws"][l], data["bs"][l]):
                params.append(dev(a)); grads.append(empty(a.shape))
                ms.append(torch.zeros(a.shape, device="cuda")); vs.append(torch.zeros(a.shape, device="cuda"))
                ref_p.append(a.astype(np.float64))
        ref_m = [np.zeros(a.shape) for a in ref_p]; ref_v = [np.zeros(a.shape) for a in ref_p]
        x, labels = dev(data["x"]), dev(data["labels"])
        opt = B.make_optimizer(B.RAD_ADAM, 1e-3, 1e-4)
        losses, ref_losses = [], []
        for t in range(1, 4):
            losses.append(B.rad_train_step(ctx, model, B.make_sampling(B.RAD_FIXEDK_PER_EXAMPLE, 0.1, t, 10, 0), x, labels,
                                           params, grads))
            B.rad_optimizer_step(ctx, opt, t, B.RAD_F32, params, grads, ms, vs)
            Ws = [ref_p[2 * l].astype(np.float32) for l in range(L)]; bs = [ref_p[2 * l + 1].astype(np.float32) for l in range(L)]
            ref = R.mlp_train_step(data["x"], data["labels"], Ws, bs, B.RAD_FIXEDK_PER_EXAMPLE, 0.1, t, stream_base=10)
            ref_losses.append(ref["loss"])
            for l in range(L):
                for j, gname in ((0, "dW"), (1, "db")):
                    i = 2 * l + j
                    ref_p[i], ref_m[i], ref_v[i] = R.adam_step(ref_p[i].astype(np.float32), ref[gname][l], ref_m[i], ref_v[i],
                                                                t, 1e-3, l2=1e-4)
        B.rad_ctx_synchronize(ctx)
        print("losses", losses, ref_losses, flush=True)
        assert np.allclose(losses, ref_losses, rtol=1e-4)
        for i in range(2 * L):
            # the first Adam steps move every weight by about lr whatever the size of its gradient, so compare
            # the movement; entries whose gradient is within rounding of zero may step the other way
            moved = host(params[i]) - (data["Ws"][i // 2] if i % 2 == 0 else data["bs"][i // 2])
            want = ref_p[i] - (data["Ws"][i // 2] if i % 2 == 0 else data["bs"][i // 2])
            assert rel_err(moved, want) < 2e-2, (i, rel_err(moved, want))
    finally:
        B.rad_model_destroy(model)

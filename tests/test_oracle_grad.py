"""Pins for the oracle's arithmetic: at fraction 1.0 (without replacement) RAD
is the baseline (Appendix A, fraction-sweep caption), so every gradient must
equal what torch's CPU autograd gives in fp64; at fraction < 1 the estimator
must be unbiased (Section 3.2, E[P] = I) with the variance its definition
implies; dX never depends on the sample (Section 4.2)."""
import numpy as np
import pytest
import torch

from oracle import rad_oracle as R


def _mlp_inputs(rng, B, dims):
    x = rng.random((B, dims[0])).astype(np.float32)
    x *= rng.random(x.shape) > 0.8
    Ws = [(rng.standard_normal((dims[i], dims[i + 1])) / np.sqrt(dims[i])).astype(np.float32)
          for i in range(len(dims) - 1)]
    bs = [(0.1 * rng.standard_normal(dims[i + 1])).astype(np.float32) for i in range(len(dims) - 1)]
    labels = rng.integers(0, dims[-1], B)
    return x, Ws, bs, labels


def _torch_mlp(x, Ws, bs, labels):
    tW = [torch.tensor(W, dtype=torch.float64, requires_grad=True) for W in Ws]
    tb = [torch.tensor(b, dtype=torch.float64, requires_grad=True) for b in bs]
    a = torch.tensor(x, dtype=torch.float64)
    for l in range(len(Ws)):
        a = a @ tW[l] + tb[l]
        if l < len(Ws) - 1:
            a = torch.relu(a)
    loss = torch.nn.functional.cross_entropy(a, torch.tensor(labels))
    loss.backward()
    return loss.item(), [w.grad.numpy() for w in tW], [b.grad.numpy() for b in tb]


@pytest.mark.parametrize("scheme", [R.EXACT, R.BERNOULLI, R.FIXEDK_SHARED, R.FIXEDK_PER_EXAMPLE])
def test_mlp_fraction_one_is_autograd(scheme):
    rng = np.random.default_rng(7)
    x, Ws, bs, labels = _mlp_inputs(rng, 23, [37, 29, 31, 10])
    out = R.mlp_train_step(x, labels, Ws, bs, scheme, 1.0, seed=5)
    loss, dW, db = _torch_mlp(x, Ws, bs, labels)
    # layer outputs are rounded to fp32 between layers: 1e-6 is that rounding
    assert abs(out["loss"] - loss) < 1e-6
    for l in range(3):
        np.testing.assert_allclose(out["dW"][l], dW[l], rtol=0, atol=2e-7)
        np.testing.assert_allclose(out["db"][l], db[l], rtol=0, atol=2e-7)


def test_single_layer_dW_dX_textbook():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((9, 6)).astype(np.float32)
    W = rng.standard_normal((6, 4)).astype(np.float32)
    dy = rng.standard_normal((9, 4)).astype(np.float32)
    h, y, bits = R.linear_forward(x, W, None, relu=True)
    tx = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    tW = torch.tensor(W, dtype=torch.float64, requires_grad=True)
    ty = torch.relu(tx @ tW)
    ty.backward(torch.tensor(dy, dtype=torch.float64))
    np.testing.assert_allclose(y, ty.detach().numpy().astype(np.float32))
    np.testing.assert_allclose(R.backward_dW(x, dy, bits), tW.grad.numpy(), atol=1e-12)
    np.testing.assert_allclose(R.backward_dX(dy, bits, W), tx.grad.numpy(), atol=1e-12)
    # transposed-operand mistakes change shapes or values; asymmetry 9x6x4 catches them


def test_relu_bit_is_strict():
    x = np.array([[1.0, -1.0]], dtype=np.float32)
    W = np.array([[1.0, 1.0, 2.0], [1.0, 2.0, 1.0]], dtype=np.float32)   # h = [0, -1, 1]
    h, y, bits = R.linear_forward(x, W, None, relu=True)
    assert list(bits[0]) == [False, False, True] and list(y[0]) == [0.0, 0.0, 1.0]


def _exact_dW(x, dy, bits):
    return x.astype(np.float64).T @ (dy.astype(np.float64) * bits)


@pytest.mark.parametrize("scheme", [R.BERNOULLI, R.FIXEDK_PER_EXAMPLE, R.FIXEDK_SHARED])
def test_unbiased_and_variance_closed_form(scheme):
    rng = np.random.default_rng(11)
    B, D, N, p, S = 12, 40, 5, 0.25, 6000
    x = rng.standard_normal((B, D)).astype(np.float32)
    dy = rng.standard_normal((B, N)).astype(np.float32)
    bits = rng.random((B, N)) > 0.4
    exact = _exact_dW(x, dy, bits)
    acc = np.zeros_like(exact)
    acc2 = np.zeros_like(exact)
    for s in range(S):
        xt = R.sample_pack(x, scheme, p, s, 1, 0)[3]
        e = R.backward_dW(xt, dy, bits)
        acc += e
        acc2 += e * e
    mean = acc / S
    var = acc2 / S - mean**2
    g2 = (dy.astype(np.float64) * bits) ** 2
    if scheme == R.FIXEDK_SHARED:
        pi = R.fixed_k(p, D) / D
        var_cf = (1 / pi - 1) * exact**2             # whole row of dW kept or dropped
    else:
        pi = p if scheme == R.BERNOULLI else R.fixed_k(p, D) / D
        var_cf = (1 / pi - 1) * (x.astype(np.float64) ** 2).T @ g2
    err = np.linalg.norm(mean - exact)
    assert err < 4 * np.sqrt(var_cf.sum() / S), (err, np.sqrt(var_cf.sum() / S))
    # the estimator is not accidentally exact, and its spread is the predicted one
    assert err > 0
    assert abs(var.sum() / var_cf.sum() - 1) < 0.08


def test_shared_scheme_leaves_unsampled_rows_zero():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((8, 50)).astype(np.float32) + 3
    dy = rng.standard_normal((8, 6)).astype(np.float32)
    bits = np.ones((8, 6), dtype=bool)
    m = R.keep_mask(R.FIXEDK_SHARED, 0.2, 9, 0, 0, 8, 50)
    dW = R.backward_dW(R.sample_pack(x, R.FIXEDK_SHARED, 0.2, 9, 0, 0)[3], dy, bits)
    assert np.all(dW[~m[0]] == 0) and np.all(np.abs(dW[m[0]]).sum(axis=1) > 0)


def test_dX_chain_independent_of_sampling():
    rng = np.random.default_rng(4)
    x, Ws, bs, labels = _mlp_inputs(rng, 10, [20, 16, 12, 5])
    ref = R.mlp_train_step(x, labels, Ws, bs, R.EXACT, 1.0, seed=0)
    for scheme, p, seed in [(R.BERNOULLI, 0.1, 1), (R.FIXEDK_PER_EXAMPLE, 0.3, 2), (R.FIXEDK_SHARED, 0.5, 3)]:
        out = R.mlp_train_step(x, labels, Ws, bs, scheme, p, seed=seed)
        assert out["loss"] == ref["loss"]
        for l in range(3):
            assert np.array_equal(out["dy"][l], ref["dy"][l])
            assert np.array_equal(out["db"][l], ref["db"][l])


def test_softmax_ce_closed_forms():
    z = np.zeros((4, 10))
    loss, dz = R.softmax_ce(z, np.array([0, 3, 5, 9]))
    assert abs(loss - np.log(10)) < 1e-15
    assert abs(dz[0, 0] - (0.1 - 1) / 4) < 1e-15 and abs(dz[0, 1] - 0.1 / 4) < 1e-15
    big = np.array([[1000.0, 0.0], [-1000.0, 0.0]])          # no overflow
    loss, dz = R.softmax_ce(big, np.array([0, 0]))
    assert abs(loss - 500.0) < 1e-9 and np.all(np.isfinite(dz))


# ------------------------------------------------------------------ conv / pool
def test_conv_pool_fraction_one_is_autograd():
    rng = np.random.default_rng(21)
    B = 3
    x = rng.standard_normal((B, 3, 8, 8)).astype(np.float32)
    shapes = [(3, 4), (4, 6), (6, 5)]
    convs, tconv = [], []
    for i, (ci, co) in enumerate(shapes):
        W = (rng.standard_normal((ci, 3, 3, co)) / np.sqrt(9 * ci)).astype(np.float32)
        b = (0.1 * rng.standard_normal(co)).astype(np.float32)
        convs.append(dict(W=W, b=b, pad=1, pool=(i >= 1)))
    fcW = (rng.standard_normal((5 * 2 * 2, 10)) / 4).astype(np.float32)
    fcb = (0.1 * rng.standard_normal(10)).astype(np.float32)
    labels = rng.integers(0, 10, B)
    out = R.cnn_train_step(x, labels, convs, (fcW, fcb), R.FIXEDK_PER_EXAMPLE, 1.0, seed=1)

    a = torch.tensor(x, dtype=torch.float64)
    tws, tbs = [], []
    for cv in convs:
        # [ci,kh,kw,co] -> torch's [co,ci,kh,kw]
        w = torch.tensor(cv["W"].transpose(3, 0, 1, 2).copy(), dtype=torch.float64, requires_grad=True)
        b = torch.tensor(cv["b"], dtype=torch.float64, requires_grad=True)
        tws.append(w); tbs.append(b)
        a = torch.relu(torch.nn.functional.conv2d(a, w, b, padding=1))
        if cv["pool"]:
            a = torch.nn.functional.max_pool2d(a, 2)
    tfw = torch.tensor(fcW, dtype=torch.float64, requires_grad=True)
    tfb = torch.tensor(fcb, dtype=torch.float64, requires_grad=True)
    z = a.reshape(B, -1) @ tfw + tfb
    loss = torch.nn.functional.cross_entropy(z, torch.tensor(labels))
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-6
    np.testing.assert_allclose(out["dW_fc"], tfw.grad.numpy(), atol=1e-6)
    np.testing.assert_allclose(out["db_fc"], tfb.grad.numpy(), atol=1e-6)
    for l in range(3):
        np.testing.assert_allclose(out["dW"][l], tws[l].grad.numpy().transpose(1, 2, 3, 0), atol=1e-6)
        np.testing.assert_allclose(out["db"][l], tbs[l].grad.numpy(), atol=1e-6)


def test_paper_convnet_shape_with_average_pool_is_autograd():
    """The convolutional architecture of Appendix A at reduced width: 5x5 convolutions with 2 zero padding,
    average pools after the second and fourth, one linear layer; at fraction 1 the oracle's step is the exact
    gradient, compared with torch's CPU autograd through avg_pool2d."""
    rng = np.random.default_rng(22)
    B = 2
    x = rng.standard_normal((B, 3, 8, 8)).astype(np.float32)
    shapes = [(3, 4), (4, 5), (5, 5), (5, 6)]
    pools = [0, 2, 0, 2]
    convs = []
    for (ci, co), pl in zip(shapes, pools):
        W = (rng.standard_normal((ci, 5, 5, co)) / np.sqrt(25 * ci)).astype(np.float32)
        b = (0.1 * rng.standard_normal(co)).astype(np.float32)
        convs.append(dict(W=W, b=b, pad=2, pool=pl))
    fcW = (rng.standard_normal((6 * 2 * 2, 10)) / 4).astype(np.float32)
    fcb = (0.1 * rng.standard_normal(10)).astype(np.float32)
    labels = rng.integers(0, 10, B)
    out = R.cnn_train_step(x, labels, convs, (fcW, fcb), R.FIXEDK_PER_EXAMPLE, 1.0, seed=1)
    a = torch.tensor(x, dtype=torch.float64)
    tws, tbs = [], []
    for cv in convs:
        w = torch.tensor(cv["W"].transpose(3, 0, 1, 2).copy(), dtype=torch.float64, requires_grad=True)
        b = torch.tensor(cv["b"], dtype=torch.float64, requires_grad=True)
        tws.append(w); tbs.append(b)
        a = torch.relu(torch.nn.functional.conv2d(a, w, b, padding=2))
        if cv["pool"] == 2:
            a = torch.nn.functional.avg_pool2d(a, 2)
            # the oracle hands fp32 activations from layer to layer
            a = a + (a.detach().to(torch.float32).to(torch.float64) - a.detach())
    tfw = torch.tensor(fcW, dtype=torch.float64, requires_grad=True)
    tfb = torch.tensor(fcb, dtype=torch.float64, requires_grad=True)
    z = a.reshape(B, -1) @ tfw + tfb
    loss = torch.nn.functional.cross_entropy(z, torch.tensor(labels))
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-6
    np.testing.assert_allclose(out["dW_fc"], tfw.grad.numpy(), atol=1e-6)
    for l in range(4):
        np.testing.assert_allclose(out["dW"][l], tws[l].grad.numpy().transpose(1, 2, 3, 0), atol=1e-6)
        np.testing.assert_allclose(out["db"][l], tbs[l].grad.numpy(), atol=1e-6)


def test_average_pool_closed_forms():
    a = np.arange(16, dtype=np.float64).reshape(1, 1, 4, 4)
    out = R.avgpool2x2_forward(a)
    assert out.tolist() == [[[[2.5, 4.5], [10.5, 12.5]]]]          # (0+1+4+5)/4, (2+3+6+7)/4, ...
    back = R.avgpool2x2_backward(np.array([[[[4.0, 8.0]]]]))
    assert back.tolist() == [[[[1.0, 1.0, 2.0, 2.0], [1.0, 1.0, 2.0, 2.0]]]]


def test_maxpool_first_max_and_zero_window():
    a = np.zeros((1, 1, 2, 4), dtype=np.float32)
    a[0, 0, :, 2:] = [[1.0, 5.0], [5.0, 2.0]]              # tie between (0,1) and (1,0)
    out, arg = R.maxpool2x2_forward(a)
    assert list(out[0, 0, 0]) == [0.0, 5.0] and list(arg[0, 0, 0]) == [0, 1]
    back = R.maxpool2x2_backward(np.array([[[[7.0, 3.0]]]]), arg)
    assert back[0, 0, 0, 0] == 7.0 and back[0, 0, 0, 3] == 3.0 and back.sum() == 10.0


def test_conv_unbiased():
    rng = np.random.default_rng(5)
    xs = rng.standard_normal((2, 2, 5, 5)).astype(np.float32)
    g = rng.standard_normal((2, 3, 5, 5))
    exact = R.conv2d_dW(xs, g, 3, 3, 1)
    acc = np.zeros_like(exact)
    S, p = 3000, 0.3
    for s in range(S):
        xt = R.sample_pack(xs.reshape(2, -1), R.BERNOULLI, p, s, 0, 0)[3].reshape(xs.shape)
        acc += R.conv2d_dW(xt, g, 3, 3, 1)
    # Var of each term x*g is (1/p - 1) x^2 g^2; sum over the terms of every dW entry
    xp = np.zeros((2, 2, 7, 7)); xp[:, :, 1:6, 1:6] = xs.astype(np.float64) ** 2
    var = 0.0
    for u in range(3):
        for v in range(3):
            var += np.einsum("bcyx,boyx->", xp[:, :, u:u + 5, v:v + 5], g**2)
    var *= (1 / p - 1)
    # terms sharing one x entry are correlated, so allow the bound a factor 9 (3x3 reuse)
    assert np.linalg.norm(acc / S - exact) < 4 * np.sqrt(9 * var / S)


# ------------------------------------------------------------------------- RNN
def _rnn_inputs(rng, B, T, H, identity=True):
    x = rng.random((B, T, 1)).astype(np.float32)
    W_ih = (np.sqrt(0.001) * rng.standard_normal((1, H))).astype(np.float32)
    W_hh = np.eye(H, dtype=np.float32) if identity else \
        (rng.standard_normal((H, H)) / np.sqrt(H)).astype(np.float32)
    b = np.zeros(H, dtype=np.float32) if identity else (0.1 * rng.standard_normal(H)).astype(np.float32)
    W_ho = (np.sqrt(0.001) * rng.standard_normal((H, 10))).astype(np.float32)
    b_o = np.zeros(10, dtype=np.float32)
    labels = rng.integers(0, 10, B)
    return x, W_ih, W_hh, b, W_ho, b_o, labels


def test_rnn_fraction_one_is_autograd():
    rng = np.random.default_rng(8)
    x, W_ih, W_hh, b, W_ho, b_o, labels = _rnn_inputs(rng, 4, 12, 9, identity=False)
    out = R.rnn_train_step(x, labels, W_ih, W_hh, b, W_ho, b_o, R.FIXEDK_PER_EXAMPLE, 1.0, seed=3)
    t = {k: torch.tensor(v, dtype=torch.float64, requires_grad=True)
         for k, v in dict(W_ih=W_ih, W_hh=W_hh, b=b, W_ho=W_ho, b_o=b_o).items()}
    h = torch.zeros(4, 9, dtype=torch.float64)
    tx = torch.tensor(x, dtype=torch.float64)
    for s in range(12):
        h = torch.relu(tx[:, s, :] @ t["W_ih"] + h @ t["W_hh"] + t["b"])
    z = h @ t["W_ho"] + t["b_o"]
    loss = torch.nn.functional.cross_entropy(z, torch.tensor(labels))
    loss.backward()
    assert abs(out["loss"] - loss.item()) < 1e-6
    for name, key in [("W_hh", "dW_hh"), ("W_ih", "dW_ih"), ("b", "db"), ("W_ho", "dW_ho"), ("b_o", "db_o")]:
        np.testing.assert_allclose(out[key], t[name].grad.numpy(), atol=1e-6, err_msg=name)


def test_rnn_identity_closed_form_forward():
    # W_hh = I, b = 0, x >= 0: units with W_ih > 0 hold W_ih * (running sum of x),
    # units with W_ih <= 0 stay at zero (Appendix A: identity initialisation).
    rng = np.random.default_rng(9)
    x, W_ih, W_hh, b, W_ho, b_o, labels = _rnn_inputs(rng, 3, 30, 16, identity=True)
    out = R.rnn_train_step(x, labels, W_ih, W_hh, b, W_ho, b_o, R.BERNOULLI, 0.1, seed=1)
    want = np.maximum(W_ih[0], 0)[None, :] * x[:, :, 0].sum(axis=1, keepdims=True)
    np.testing.assert_allclose(out["h_T"], want, rtol=1e-5)


def test_rnn_unbiased_dW_hh():
    rng = np.random.default_rng(10)
    x, W_ih, W_hh, b, W_ho, b_o, labels = _rnn_inputs(rng, 3, 6, 8, identity=False)
    exact = R.rnn_train_step(x, labels, W_ih, W_hh, b, W_ho, b_o, R.EXACT, 1.0, seed=0)
    acc = np.zeros_like(exact["dW_hh"]); acc2 = np.zeros_like(acc)
    S = 2000
    for s in range(S):
        o = R.rnn_train_step(x, labels, W_ih, W_hh, b, W_ho, b_o, R.BERNOULLI, 0.3, seed=s)
        acc += o["dW_hh"]; acc2 += o["dW_hh"] ** 2
        assert np.array_equal(o["dW_ih"], exact["dW_ih"])      # unsampled paths are exact
    var = acc2 / S - (acc / S) ** 2
    assert np.linalg.norm(acc / S - exact["dW_hh"]) < 4 * np.sqrt(var.sum() / S)

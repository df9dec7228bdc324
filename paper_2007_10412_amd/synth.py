"""Seeded synthetic inputs with the shapes and value statistics of the paper's
workloads (MNIST-like sparse pixels, CIFAR-like normal images, sequential
MNIST).  Holds no arithmetic of the method: the CPU reference used by the tests and the
HIP path are fed from here with identical host arrays."""
import numpy as np


def bf16_round(a):
    """float32 array rounded to bfloat16-representable values (via torch's cast)."""
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(torch.bfloat16).to(torch.float32).numpy()


def sparse_pixels(rng, batch, d):
    """uniform[0,1) with 80 % of the entries zeroed: stands in for MNIST pixels."""
    x = rng.random((batch, d), dtype=np.float32)
    x *= rng.random((batch, d)) >= 0.8
    return x.astype(np.float32)


def weight(rng, d_in, d_out):
    """N(0, 1/d_in), in x out layout."""
    return (rng.standard_normal((d_in, d_out)) / np.sqrt(d_in)).astype(np.float32)


def single_layer(seed=1234, batch=150, d_in=784, d_out=300):
    """Config 1: x [150,784] sparse pixels, W ~ N(0,1/784), upstream dy ~ N(0, 0.01)."""
    rng = np.random.default_rng(seed)
    return dict(x=sparse_pixels(rng, batch, d_in), W=weight(rng, d_in, d_out),
                dy=(0.1 * rng.standard_normal((batch, d_out))).astype(np.float32))


def mlp(seed=1234, batch=150, dims=(784, 300, 300, 10), pixels=True, bias_scale=0.0, bf16=False):
    """Configs 2 and 4: MLP inputs, weights N(0,1/fan_in), biases (zero unless bias_scale), labels."""
    rng = np.random.default_rng(seed)
    x = sparse_pixels(rng, batch, dims[0]) if pixels else rng.standard_normal((batch, dims[0])).astype(np.float32)
    Ws = [weight(rng, dims[i], dims[i + 1]) for i in range(len(dims) - 1)]
    bs = [(bias_scale * rng.standard_normal(dims[i + 1])).astype(np.float32) for i in range(len(dims) - 1)]
    labels = rng.integers(0, dims[-1], batch).astype(np.int32)
    if bf16:
        x = bf16_round(x)
        Ws = [bf16_round(W) for W in Ws]
    return dict(x=x, Ws=Ws, bs=bs, labels=labels)


def rnn(seed=1234, batch=128, T=784, d_input=1, hidden=1024, classes=10, identity=True):
    """Config 5: sequential-MNIST-like pixels in [0,1), W_hh = I, W_ih and W_ho ~ N(0, 0.001), zero biases."""
    rng = np.random.default_rng(seed)
    x = rng.random((batch, T, d_input), dtype=np.float32)
    std = np.sqrt(0.001)
    W_ih = (std * rng.standard_normal((d_input, hidden))).astype(np.float32)
    W_hh = np.eye(hidden, dtype=np.float32) if identity else weight(rng, hidden, hidden)
    b = np.zeros(hidden, dtype=np.float32) if identity else (0.1 * rng.standard_normal(hidden)).astype(np.float32)
    W_ho = (std * rng.standard_normal((hidden, classes))).astype(np.float32)
    b_o = np.zeros(classes, dtype=np.float32)
    labels = rng.integers(0, classes, batch).astype(np.int32)
    return dict(x=x, W_ih=W_ih, W_hh=W_hh, b=b, W_ho=W_ho, b_o=b_o, labels=labels)


def cnn(seed=1234, batch=150, channels=(3, 16, 32, 64), pool=(0, 1, 1), ksize=3, hw=32, classes=10):
    """Config 3: N(0,1) images, conv weights [c_in,k,k,c_out] ~ N(0, 1/(c_in k k)), zero biases.
    pool[i]: 0 none, 1 max pool, 2 average pool after conv i."""
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((batch, channels[0], hw, hw)).astype(np.float32)
    convs = []
    size = hw
    for i in range(len(channels) - 1):
        ci, co = channels[i], channels[i + 1]
        W = (rng.standard_normal((ci, ksize, ksize, co)) / np.sqrt(ci * ksize * ksize)).astype(np.float32)
        convs.append(dict(W=W, b=np.zeros(co, dtype=np.float32), pad=(ksize - 1) // 2, pool=int(pool[i])))
        if pool[i]:
            size //= 2
    d = channels[-1] * size * size
    fc = (weight(rng, d, classes), np.zeros(classes, dtype=np.float32))
    labels = rng.integers(0, classes, batch).astype(np.int32)
    return dict(x=x, convs=convs, fc=fc, labels=labels)

"""CPU oracle for the Randomized-AD (RAD) linear-layer training step.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition of what the
HIP library computes.  Only tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py may import it.  It shares no code with the HIP
path and never imports it.

Everything floating point accumulates in fp64 (numpy matmul / einsum as the
library primitive); values are rounded to the storage dtype (fp32, or bf16 with
round-to-nearest-even) exactly at the places a layer output or a stored sample
leaves a kernel.  Integer work (keys, selection, indices) is exact.

Notation follows the paper (Section 3.2 and Section 4.2): a linear layer has
input x [B, D], weight W [D, N], pre-activation h = x W + b, activation
y = ReLU(h); the upstream gradient is dy = dL/dy, g = dy * 1[h > 0].  RAD
replaces the stored x by x~ = x P with E[P] = I_D (Section 3.2, the random
matrix P), so that dW~ = x~^T g is an unbiased estimate of dW = x^T g, while
dX = g W^T never touches a sampled quantity (Section 4.2: only dh/dW is
sampled, so every parameter-to-loss path crosses one sampled Jacobian).

The with-replacement schemes are the matrix P of Section 3.2 as printed:
P = (d/k) sum_s e_{i_s} e_{i_s}^T with k indices i_s drawn uniformly and
independently, so coordinate j carries the weight m_j d/k, m_j being how often j
was drawn (pins: multiplicities sum to k and are Binomial(k, 1/d); the
closed-form variance ((d-1)/k) sum_b x^2 g^2; k = d does not give the baseline).

The projection scheme is the other P of Section 3.2 / Appendix "Random
projections for RAD": P = R R^T / k with R [d, k] independent signs, so the
store is z = x R / sqrt(k) (k numbers per row, no indices) and the backward
pass uses x~ = z R^T / sqrt(k) (pins: E[P] = I, the closed-form variance
(|dW[:, n]|^2 - dW[j, n]^2) / k, sign balance and independence).

Pins (tests/test_oracle_*.py): Philox against PyTorch's own Philox4_32 engine;
k = ceil(p d) against the eight worked values of Appendix A; byte accounting
against Appendix A and Table 1; p = 1 against torch autograd; mean and variance
over seeds against closed forms; selection against brute force; the optimiser
steps against torch.optim on the CPU and a closed form.  Convergence
curves of the paper (figures only) are not reproducible: parity unpinned there.
"""
from __future__ import annotations

import math

import numpy as np

# ----------------------------------------------------------------------------
# Sampling schemes (values are part of the C ABI; the oracle repeats them).
# ----------------------------------------------------------------------------
EXACT = 0               # store everything (the paper's baseline)
BERNOULLI = 1           # keep each entry with probability p, scale 1/p
FIXEDK_SHARED = 2       # "same sample": one k-subset for the whole minibatch
FIXEDK_PER_EXAMPLE = 3  # "different sample": a k-subset per minibatch element
REPLACE_SHARED = 4      # k draws WITH replacement, one set for the whole minibatch
REPLACE_PER_EXAMPLE = 5  # k draws WITH replacement per minibatch element
PROJECT_SHARED = 6      # "project": x R / sqrt(k) with one Rademacher matrix R [d, k]
PROJECT_PER_EXAMPLE = 7  # "different project": a Rademacher matrix of its own for every example

F32 = 0
BF16 = 1

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK32 = np.uint64(0xFFFFFFFF)


# ----------------------------------------------------------------------------
# Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as easy
# as 1, 2, 3", SC'11).  The paper names no generator; a counter-based one makes
# the sample a pure function of (seed, tensor, step, element).
# ----------------------------------------------------------------------------
def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Ten Philox rounds on arrays of 32-bit counter words; returns 4 arrays."""
    c0 = np.asarray(c0, dtype=np.uint64)
    c1 = np.asarray(c1, dtype=np.uint64)
    c2 = np.asarray(c2, dtype=np.uint64)
    c3 = np.asarray(c3, dtype=np.uint64)
    k0 = int(k0) & 0xFFFFFFFF
    k1 = int(k1) & 0xFFFFFFFF
    for r in range(10):
        if r > 0:
            k0 = (k0 + _W0) & 0xFFFFFFFF
            k1 = (k1 + _W1) & 0xFFFFFFFF
        p0 = _M0 * c0          # 32x32 -> 64 bit product, exact in uint64
        p1 = _M1 * c2
        hi0, lo0 = p0 >> np.uint64(32), p0 & _MASK32
        hi1, lo1 = p1 >> np.uint64(32), p1 & _MASK32
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1,
                          hi0 ^ c3 ^ np.uint64(k1), lo0)
    return (c0.astype(np.uint32), c1.astype(np.uint32),
            c2.astype(np.uint32), c3.astype(np.uint32))


def element_keys(seed, stream_id, step, first, count):
    """One u32 key for each flat element index f in [first, first+count).

    Addressing (the paper is silent; this is the library's definition):
    Philox key = (seed low word, seed high word); counter =
    (floor(f/4) low word, floor(f/4) high word, stream_id, step); the element
    takes output word f mod 4.  Keys therefore depend on nothing but
    (seed, stream_id, step, f).
    """
    f = np.arange(first, first + count, dtype=np.uint64)
    q = f >> np.uint64(2)
    w = (f & np.uint64(3)).astype(np.int64)
    out = philox4x32_10(q & _MASK32, q >> np.uint64(32),
                        np.uint64(stream_id & 0xFFFFFFFF),
                        np.uint64(step & 0xFFFFFFFF),
                        seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    stacked = np.stack(out, axis=-1)
    return np.take_along_axis(stacked, w[:, None], axis=1)[:, 0]


# ----------------------------------------------------------------------------
# Selection rules.
# ----------------------------------------------------------------------------
def fixed_k(p, d):
    """Number of stored coordinates: p*d rounded up (Appendix A, memory
    calculation), kept inside [1, d].  The 1e-9 guards products such as
    0.1*300 that land an ulp above an integer in binary floating point."""
    return int(min(d, max(1, math.ceil(p * d - 1e-9))))


def bernoulli_threshold(p):
    """Keep iff key < T with T = round(p * 2^32) held in 64 bits (p = 1 keeps
    every key)."""
    return int(round(p * 4294967296.0))


def sample_scale(scheme, p, d):
    """Inverse inclusion probability, as fp32.  Bernoulli: 1/p.  Fixed-k
    (with or without replacement): d/k (Section 3.2 scales by d/k)."""
    if scheme == EXACT:
        return np.float32(1.0)
    if scheme == BERNOULLI:
        return np.float32(1.0 / p)
    return np.float32(float(d) / float(fixed_k(p, d)))


def replace_draws(scheme, p, seed, stream_id, step, rows, d):
    """Indices i_s of the k uniform draws with replacement (Section 3.2: each
    P_s is sampled uniformly from {P_1 .. P_d}), [rows, k].

    Draw s of row b takes the key of flat index f = b k + s (f = s for the
    shared scheme) in the element_keys addressing and maps it to
    i = floor(key * d / 2^32): every index owns floor or ceil of 2^32/d keys.
    """
    k = fixed_k(p, d)
    if scheme == REPLACE_SHARED:
        keys = element_keys(seed, stream_id, step, 0, k).reshape(1, k)
    elif scheme == REPLACE_PER_EXAMPLE:
        keys = element_keys(seed, stream_id, step, 0, rows * k).reshape(rows, k)
    else:
        raise ValueError("not a with-replacement scheme")
    idx = (keys.astype(np.uint64) * np.uint64(d)) >> np.uint64(32)
    if scheme == REPLACE_SHARED:
        idx = np.broadcast_to(idx, (rows, k))
    return idx.astype(np.int64)


def multiplicity(scheme, p, seed, stream_id, step, rows, d):
    """m [rows, d]: how often each coordinate was drawn; rows sum to k."""
    idx = replace_draws(scheme, p, seed, stream_id, step, rows, d)
    m = np.zeros((rows, d), dtype=np.int64)
    for b in range(rows):
        np.add.at(m[b], idx[b], 1)
    return m


def rademacher_matrix(p, seed, stream_id, step, d):
    """R [d, k] with entries +1 / -1 (Appendix, random projections: a matrix of
    independent Rademacher variables).  Entry (j, s) takes bit (f mod 32) of
    the key of flat index floor(f / 32), f = j k + s, in the element_keys
    addressing; a clear bit is +1, a set bit -1.
    """
    k = fixed_k(p, d)
    n = d * k
    words = element_keys(seed, stream_id, step, 0, (n + 31) // 32)
    f = np.arange(n, dtype=np.int64)
    bit = (words[f >> 5] >> (f & 31).astype(np.uint32)) & np.uint32(1)
    return (1.0 - 2.0 * bit.astype(np.float64)).reshape(d, k)


def rademacher_matrix_of_example(p, seed, stream_id, step, b, d):
    """R_b [d, k] for example b ("different project", Appendix A, RNN
    experiments: a different random matrix for each mini-batch element).  Row
    (b, j) of the sign tensor owns the 4 C consecutive keys that start at flat
    index (b d + j) 4 C, C = ceil(k / 128), i.e. whole Philox calls; sign s is
    bit s mod 32 of the row's key number s div 32; clear is +1, set is -1.
    """
    k = fixed_k(p, d)
    words_per_row = 4 * ((k + 127) // 128)
    words = element_keys(seed, stream_id, step, b * d * words_per_row, d * words_per_row)
    words = words.reshape(d, words_per_row)
    sidx = np.arange(k)
    bit = (words[:, sidx >> 5] >> (sidx & 31).astype(np.uint32)[None, :]) & np.uint32(1)
    return 1.0 - 2.0 * bit.astype(np.float64)


def project_store(x, p, seed, stream_id, step, dtype=F32, per_example=False):
    """z = storage(x R * fp32(1/sqrt(k))) [rows, k] and the backward operand
    x~ = z R^T / sqrt(k) [rows, d] (fp64), so that x~ = x P with P = R R^T / k;
    per_example: row b uses its own R_b."""
    x = np.asarray(x, dtype=np.float32)
    rows, d = x.shape
    k = fixed_k(p, d)
    inv = np.float64(np.float32(1.0 / math.sqrt(k)))
    if not per_example:
        R = rademacher_matrix(p, seed, stream_id, step, d)
        z = to_storage((x.astype(np.float64) @ R) * inv, dtype)
        xt = (z.astype(np.float64) @ R.T) * inv
        return z, xt
    z = np.zeros((rows, k), dtype=np.float32)
    xt = np.zeros((rows, d))
    for b in range(rows):
        R = rademacher_matrix_of_example(p, seed, stream_id, step, b, d)
        z[b] = to_storage((x[b].astype(np.float64) @ R) * inv, dtype)
        xt[b] = (z[b].astype(np.float64) @ R.T) * inv
    return z, xt


def keep_mask(scheme, p, seed, stream_id, step, rows, d):
    """Boolean [rows, d]: which entries of the sampled tensor are stored.

    Bernoulli: key < T.  Fixed-k: the k smallest (key, j) pairs of the row in
    lexicographic order (ties go to the lower j), i.e. a uniform k-subset
    without replacement: the variant the paper says makes fraction 1.0 equal
    to the baseline (Appendix A, fraction sweep caption).  Shared scheme: the
    keys of row 0 addressing (f = j) serve every row.
    """
    if scheme == EXACT:
        return np.ones((rows, d), dtype=bool)
    if scheme == BERNOULLI:
        keys = element_keys(seed, stream_id, step, 0, rows * d).reshape(rows, d)
        return keys.astype(np.uint64) < np.uint64(bernoulli_threshold(p))
    if scheme in (REPLACE_SHARED, REPLACE_PER_EXAMPLE):
        return multiplicity(scheme, p, seed, stream_id, step, rows, d) > 0
    k = fixed_k(p, d)
    if scheme == FIXEDK_SHARED:
        keys = element_keys(seed, stream_id, step, 0, d).reshape(1, d)
    elif scheme == FIXEDK_PER_EXAMPLE:
        keys = element_keys(seed, stream_id, step, 0, rows * d).reshape(rows, d)
    else:
        raise ValueError("unknown scheme")
    order = np.argsort(keys, axis=1, kind="stable")   # stable: ties by lower j
    mask = np.zeros(keys.shape, dtype=bool)
    np.put_along_axis(mask, order[:, :k], True, axis=1)
    if scheme == FIXEDK_SHARED:
        mask = np.broadcast_to(mask, (rows, d)).copy()
    return mask


# ----------------------------------------------------------------------------
# Storage dtype rounding.
# ----------------------------------------------------------------------------
def round_bf16(a):
    """fp32 -> bfloat16 (round to nearest, ties to even) -> fp32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32).astype(np.uint64)
    lsb = (u >> np.uint64(16)) & np.uint64(1)
    r = ((u + np.uint64(0x7FFF) + lsb) >> np.uint64(16)) << np.uint64(16)
    out = (r & _MASK32).astype(np.uint32).view(np.float32)
    return np.where(np.isnan(a), a, out).reshape(a.shape)


def to_storage(a, dtype):
    """Round an fp64/fp32 array to the storage dtype, returned as fp32."""
    a32 = np.asarray(a, dtype=np.float64).astype(np.float32)
    return round_bf16(a32) if dtype == BF16 else a32


# ----------------------------------------------------------------------------
# The compressed store.
# ----------------------------------------------------------------------------
def sample_pack(x, scheme, p, seed, stream_id, step, dtype=F32):
    """x [rows, d] (already in storage precision) -> (row_ptr, col, val, xt).

    val = storage(x * scale) for kept entries, ascending column per row; xt is
    the same thing scattered back into a dense [rows, d] array (x~ = x P of
    Section 3.2 with P diagonal).  Sampled zeros are stored like any value, so
    the size never depends on the data.
    """
    x = np.asarray(x, dtype=np.float32)
    rows, d = x.shape
    if scheme in (PROJECT_SHARED, PROJECT_PER_EXAMPLE):
        # the store is the dense projection z: listed as k "columns" 0..k-1 per row
        z, xt = project_store(x, p, seed, stream_id, step, dtype, scheme == PROJECT_PER_EXAMPLE)
        k = z.shape[1]
        row_ptr = np.arange(rows + 1, dtype=np.int64) * k
        col = np.tile(np.arange(k, dtype=np.int32), rows)
        return row_ptr, col, z.reshape(-1), xt
    scale = sample_scale(scheme, p, d)
    if scheme in (REPLACE_SHARED, REPLACE_PER_EXAMPLE):
        # weight of coordinate j is m_j d/k: the fp32 product of the count and the fp32 scale, then one fp32
        # multiply with x and one rounding (a coordinate drawn once is scaled exactly as in the other schemes)
        m = multiplicity(scheme, p, seed, stream_id, step, rows, d)
        mask = m > 0
        weight = (m.astype(np.float32) * scale).astype(np.float32)
        scaled = to_storage(x * weight, dtype)
    else:
        mask = keep_mask(scheme, p, seed, stream_id, step, rows, d)
        scaled = to_storage(x * scale, dtype)            # one fp32 multiply, one rounding
    xt = np.where(mask, scaled, np.float32(0.0))
    row_ptr = np.zeros(rows + 1, dtype=np.int64)
    row_ptr[1:] = np.cumsum(mask.sum(axis=1))
    r, c = np.nonzero(mask)                          # row-major => ascending col per row
    return row_ptr, c.astype(np.int32), scaled[r, c], xt


# ----------------------------------------------------------------------------
# Linear layer.
# ----------------------------------------------------------------------------
def linear_forward(x, W, bias, relu, dtype=F32):
    """h = x W + b with the exact x (Section 3: the forward pass is the
    original graph); returns (h fp64, y storage-rounded fp32, bits bool).
    The ReLU Jacobian is one bit per entry (Section 4.2): bits = h > 0."""
    h = np.asarray(x, dtype=np.float64) @ np.asarray(W, dtype=np.float64)
    if bias is not None:
        h = h + np.asarray(bias, dtype=np.float64)[None, :]
    if relu:
        bits = h > 0.0
        y = np.where(bits, h, 0.0)
    else:
        bits = np.ones(h.shape, dtype=bool)
        y = h
    return h, to_storage(y, dtype), bits


def backward_dW(xt, dy, bits):
    """dW~ = x~^T (dy * bits): the sampled Jacobian dh/dW of Section 4.2."""
    g = np.asarray(dy, dtype=np.float64) * bits
    return np.asarray(xt, dtype=np.float64).T @ g


def backward_db(dy, bits):
    return (np.asarray(dy, dtype=np.float64) * bits).sum(axis=0)


def backward_dX(dy, bits, W):
    """dX = (dy * bits) W^T: exact, independent of p and seed."""
    g = np.asarray(dy, dtype=np.float64) * bits
    return g @ np.asarray(W, dtype=np.float64).T


# ----------------------------------------------------------------------------
# Loss: softmax cross-entropy, mean over the batch.  Logits stay dense
# (Appendix A: the softmax input is not sampled).
# ----------------------------------------------------------------------------
def softmax_ce(z, labels):
    z = np.asarray(z, dtype=np.float64)
    b = z.shape[0]
    zs = z - z.max(axis=1, keepdims=True)
    e = np.exp(zs)
    s = e.sum(axis=1, keepdims=True)
    logp = zs - np.log(s)
    loss = -logp[np.arange(b), labels].mean()
    dz = e / s
    dz[np.arange(b), labels] -= 1.0
    return loss, dz / b


# ----------------------------------------------------------------------------
# Multi-layer perceptron train step (Section 4.2, generalised chain).
# ----------------------------------------------------------------------------
def mlp_train_step(x, labels, Ws, bs, scheme, p, seed, stream_base=0, step=0,
                   dtype=F32, bits_override=None):
    """Forward with exact activations, storing for each layer only the sample
    of its input and its ReLU bits; backward from those.

    Layer l samples with stream_id = stream_base + l.  All layers but the last
    have ReLU.  Returns a dict with loss, per-layer dW/db, stores, bits,
    activations and the dy chain.  bits_override (list of bool arrays) lets a
    test rerun the backward with ReLU bits taken from elsewhere.
    """
    L = len(Ws)
    act = to_storage(x, dtype)
    stores, bits_l, acts = [], [], [act]
    for l in range(L):
        stores.append(sample_pack(act, scheme, p, seed, stream_base + l, step, dtype))
        _, y, bits = linear_forward(act, Ws[l], None if bs is None else bs[l],
                                    relu=(l < L - 1), dtype=dtype)
        if bits_override is not None and l < L - 1:
            bits = bits_override[l]
        bits_l.append(bits)
        act = y
        acts.append(act)
    loss, dz = softmax_ce(act, labels)
    dy = to_storage(dz, dtype)
    dWs, dbs, dys = [None] * L, [None] * L, [None] * L
    for l in range(L - 1, -1, -1):
        dys[l] = dy
        dWs[l] = backward_dW(stores[l][3], dy, bits_l[l])
        dbs[l] = backward_db(dy, bits_l[l])
        if l > 0:
            dy = to_storage(backward_dX(dy, bits_l[l], Ws[l]), dtype)
    return dict(loss=loss, dW=dWs, db=dbs, stores=stores, bits=bits_l,
                acts=acts, dy=dys)


# ----------------------------------------------------------------------------
# Convolution (stride 1, zero padding) written as the sum it is; weights are
# laid out [C_in, KH, KW, C_out] so that the flattened [C_in*KH*KW, C_out]
# matrix is the W of the equivalent im2col GEMM.  Activations are NCHW.
# The sampled tensor is the layer input, flattened to [B, C*H*W] (Figure 5:
# spatial elements of the input are sampled and dH/dW is formed from the
# sparse tensor).
# ----------------------------------------------------------------------------
def conv2d_forward(x, W, bias, pad, relu):
    x = np.asarray(x, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    b, ci, hh, ww = x.shape
    _, kh, kw, co = W.shape
    xp = np.zeros((b, ci, hh + 2 * pad, ww + 2 * pad))
    xp[:, :, pad:pad + hh, pad:pad + ww] = x
    ho, wo = hh + 2 * pad - kh + 1, ww + 2 * pad - kw + 1
    h = np.zeros((b, co, ho, wo))
    for u in range(kh):
        for v in range(kw):
            # h[b,o,y,x] += sum_c xp[b,c,y+u,x+v] * W[c,u,v,o]
            h += np.einsum("bcyx,co->boyx", xp[:, :, u:u + ho, v:v + wo], W[:, u, v, :])
    if bias is not None:
        h = h + np.asarray(bias, dtype=np.float64)[None, :, None, None]
    if relu:
        bits = h > 0.0
        y = np.where(bits, h, 0.0)
    else:
        bits = np.ones(h.shape, dtype=bool)
        y = h
    return h, y.astype(np.float32), bits


def conv2d_dW(xt, g, kh, kw, pad):
    """dW[c,u,v,o] = sum_{b,y,x} xt_padded[b,c,y+u,x+v] * g[b,o,y,x]."""
    xt = np.asarray(xt, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    b, ci, hh, ww = xt.shape
    co, ho, wo = g.shape[1:]
    xp = np.zeros((b, ci, hh + 2 * pad, ww + 2 * pad))
    xp[:, :, pad:pad + hh, pad:pad + ww] = xt
    dW = np.zeros((ci, kh, kw, co))
    for u in range(kh):
        for v in range(kw):
            dW[:, u, v, :] = np.einsum("bcyx,boyx->co", xp[:, :, u:u + ho, v:v + wo], g)
    return dW


def conv2d_dX(g, W, pad, in_hw):
    """dX[b,c,i,j] = sum_{o,u,v} g[b,o,i-u+pad,j-v+pad] * W[c,u,v,o]."""
    g = np.asarray(g, dtype=np.float64)
    W = np.asarray(W, dtype=np.float64)
    b, co, ho, wo = g.shape
    ci, kh, kw, _ = W.shape
    hh, ww = in_hw
    dxp = np.zeros((b, ci, hh + 2 * pad, ww + 2 * pad))
    for u in range(kh):
        for v in range(kw):
            dxp[:, :, u:u + ho, v:v + wo] += np.einsum("boyx,co->bcyx", g, W[:, u, v, :])
    return dxp[:, :, pad:pad + hh, pad:pad + ww]


def maxpool2x2_forward(a):
    """2x2/stride-2 max pool; argmax = first maximum in (dy, dx) row-major
    order, stored in 2 bits."""
    a = np.asarray(a)
    b, c, hh, ww = a.shape
    win = a.reshape(b, c, hh // 2, 2, ww // 2, 2).transpose(0, 1, 2, 4, 3, 5)
    win = win.reshape(b, c, hh // 2, ww // 2, 4)
    arg = np.argmax(win, axis=-1)          # numpy returns the first maximum
    out = np.take_along_axis(win, arg[..., None], axis=-1)[..., 0]
    return out, arg.astype(np.uint8)


def maxpool2x2_backward(dout, arg):
    dout = np.asarray(dout, dtype=np.float64)
    b, c, ho, wo = dout.shape
    win = np.zeros((b, c, ho, wo, 4))
    np.put_along_axis(win, arg[..., None].astype(np.int64), dout[..., None], axis=-1)
    win = win.reshape(b, c, ho, wo, 2, 2).transpose(0, 1, 2, 4, 3, 5)
    return win.reshape(b, c, ho * 2, wo * 2)


def avgpool2x2_forward(a):
    """2x2/stride-2 average pool (the pooling of the convolutional architecture
    in Appendix A).  Its Jacobian is constant, so nothing is kept for the
    backward pass (Appendix A, calculation of memory saved)."""
    a = np.asarray(a, dtype=np.float64)
    b, c, hh, ww = a.shape
    return a.reshape(b, c, hh // 2, 2, ww // 2, 2).mean(axis=(3, 5))


def avgpool2x2_backward(dout):
    """Every input of a window receives a quarter of the window's gradient."""
    dout = np.asarray(dout, dtype=np.float64)
    return np.repeat(np.repeat(dout, 2, axis=2), 2, axis=3) / 4.0


def cnn_train_step(x, labels, convs, fc, scheme, p, seed, stream_base=0, step=0,
                   bits_override=None, arg_override=None):
    """convs: list of dicts(W [ci,kh,kw,co], b [co], pad, pool); every conv is
    followed by ReLU and then by a 2x2 max pool if pool is 1 (or True), a 2x2
    average pool if pool is 2, nothing if 0.  fc = (W [D,10], b).
    Each conv input and the FC input is sampled (flattened per example).
    bits_override / arg_override (lists, entries may be None) replace the ReLU
    bits / pool positions used in the backward pass, for tests that feed one
    side's near-tie decisions to the other."""
    act = np.asarray(x, dtype=np.float32)
    B = act.shape[0]
    tape, stores = [], []
    for l, cv in enumerate(convs):
        st = sample_pack(act.reshape(B, -1), scheme, p, seed, stream_base + l, step)
        stores.append(st)
        _, y, bits = conv2d_forward(act, cv["W"], cv["b"], cv["pad"], relu=True)
        arg = None
        in_shape = act.shape
        kind = int(cv["pool"])
        if kind == 1:
            y, arg = maxpool2x2_forward(y)
        elif kind == 2:
            y = avgpool2x2_forward(y)
        if bits_override is not None and bits_override[l] is not None:
            bits = bits_override[l]
        if arg_override is not None and arg_override[l] is not None:
            arg = arg_override[l]
        tape.append((in_shape, bits, arg, kind))
        act = y.astype(np.float32)
    flat = act.reshape(B, -1)
    st_fc = sample_pack(flat, scheme, p, seed, stream_base + len(convs), step)
    stores.append(st_fc)
    _, z, _ = linear_forward(flat, fc[0], fc[1], relu=False)
    loss, dz = softmax_ce(z, labels)
    dz = dz.astype(np.float32)
    ones = np.ones(dz.shape, dtype=bool)
    dW_fc = backward_dW(st_fc[3], dz, ones)
    db_fc = backward_db(dz, ones)
    dy = backward_dX(dz, ones, fc[0]).astype(np.float32).reshape(act.shape)
    dWs, dbs = [None] * len(convs), [None] * len(convs)
    for l in range(len(convs) - 1, -1, -1):
        cv = convs[l]
        in_shape, bits, arg, kind = tape[l]
        if kind == 1:
            dy = maxpool2x2_backward(dy, arg)
        elif kind == 2:
            dy = avgpool2x2_backward(dy)
        g = np.asarray(dy, dtype=np.float64) * bits
        kh, kw = cv["W"].shape[1:3]
        dWs[l] = conv2d_dW(stores[l][3].reshape(in_shape), g, kh, kw, cv["pad"])
        dbs[l] = g.sum(axis=(0, 2, 3))
        if l > 0:
            dy = conv2d_dX(g, cv["W"], cv["pad"], in_shape[2:]).astype(np.float32)
    return dict(loss=loss, dW=dWs, db=dbs, dW_fc=dW_fc, db_fc=db_fc,
                stores=stores, logits=z, tape=tape)


# ----------------------------------------------------------------------------
# Vanilla ReLU RNN with BPTT (Appendix A, recurrent architecture):
# h_t = ReLU(x_t W_ih + h_{t-1} W_hh + b), t = 1..T, h_0 = 0; logits =
# h_T W_ho + b_o.  A fresh sample of h_{t-1} is stored at every time step
# (Appendix A, RNN training details); the 1-dimensional x_t is kept whole
# (ceil(0.1*1) = 1 in Appendix A's count).
# ----------------------------------------------------------------------------
def rnn_train_step(x, labels, W_ih, W_hh, b, W_ho, b_o, scheme, p, seed,
                   stream_base=0):
    """x [B, T, I].  Sampling of h_{t-1} uses stream_id = stream_base and
    step = t (t = 1..T; nothing is stored for t = 1 because h_0 = 0); the
    output layer samples h_T with stream_id = stream_base + 1, step = 0."""
    x = np.asarray(x, dtype=np.float32)
    B, T, _ = x.shape
    H = W_hh.shape[0]
    h_prev = np.zeros((B, H), dtype=np.float32)
    xts, bits_t, stores_t = [None] * (T + 1), [None] * (T + 1), [None] * (T + 1)
    W_ih64 = np.asarray(W_ih, dtype=np.float64)
    W_hh64 = np.asarray(W_hh, dtype=np.float64)
    b64 = np.asarray(b, dtype=np.float64)
    for t in range(1, T + 1):
        if t > 1:
            sp = sample_pack(h_prev, scheme, p, seed, stream_base, t)
            stores_t[t], xts[t] = sp[:3], sp[3]
        pre = (x[:, t - 1, :].astype(np.float64) @ W_ih64
               + h_prev.astype(np.float64) @ W_hh64 + b64[None, :])
        bits_t[t] = pre > 0.0
        h_prev = np.where(bits_t[t], pre, 0.0).astype(np.float32)
    st_o = sample_pack(h_prev, scheme, p, seed, stream_base + 1, 0)
    _, z, _ = linear_forward(h_prev, W_ho, b_o, relu=False)
    loss, dz = softmax_ce(z, labels)
    dz = dz.astype(np.float32)
    ones = np.ones(dz.shape, dtype=bool)
    dW_ho = backward_dW(st_o[3], dz, ones)
    db_o = backward_db(dz, ones)
    dh = backward_dX(dz, ones, W_ho).astype(np.float32)
    dW_hh = np.zeros((H, H))
    dW_ih = np.zeros(W_ih64.shape)
    db = np.zeros(H)
    for t in range(T, 0, -1):
        g = dh.astype(np.float64) * bits_t[t]
        if t > 1:
            dW_hh += xts[t].astype(np.float64).T @ g
        dW_ih += x[:, t - 1, :].astype(np.float64).T @ g
        db += g.sum(axis=0)
        dh = (g @ W_hh64.T).astype(np.float32)
    return dict(loss=loss, dW_hh=dW_hh, dW_ih=dW_ih, db=db, dW_ho=dW_ho,
                db_o=db_o, h_T=h_prev, logits=z, stores=stores_t, store_o=st_o[:3])


# ----------------------------------------------------------------------------
# Parameter updates (Section 4.3 and Appendix A, feedforward and RNN training
# details): the feedforward networks are trained with Adam, with a tuned
# learning rate and l2 regularisation coefficient; the RNN with plain SGD
# without momentum.  The l2 term enters as a gradient of (l2/2)|w|^2, i.e.
# g + l2 w (a reading: the paper names the coefficient, not the form).  Adam is
# the algorithm the paper cites (Kingma & Ba 2015, Algorithm 1): exponential
# moving averages of g and g^2, both divided by 1 - beta^t, step
# lr m^ / (sqrt(v^) + eps).  Learning-rate schedules (Appendix A multiplies the
# rate by 0.6 at fixed intervals) belong to the caller, who passes lr per step.
# Pins (tests/test_oracle_optim.py): torch.optim's CPU SGD and Adam, and the
# closed form under a constant gradient.
# ----------------------------------------------------------------------------
def sgd_step(w, g, lr, l2=0.0):
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64) + l2 * w
    return w - lr * g


def adam_step(w, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, l2=0.0):
    """Step number t (1, 2, ...) from moments m, v (zeros before step 1);
    returns the new (w, m, v), all float64."""
    w = np.asarray(w, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64) + l2 * w
    m = beta1 * np.asarray(m, dtype=np.float64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, dtype=np.float64) + (1.0 - beta2) * g * g
    m_hat = m / (1.0 - beta1 ** t)
    v_hat = v / (1.0 - beta2 ** t)
    return w - lr * m_hat / (np.sqrt(v_hat) + eps), m, v


# ----------------------------------------------------------------------------
# Reaction-diffusion PDE-constrained optimisation (Section 5, Appendix B).
# phi lives on the nodes (i, j), 0 <= i, j <= n, of the unit square (x = i/n,
# y = j/n) and is zero on the boundary; the explicit update of Appendix B is
#   phi_{t+1} = phi_t + (D dt / dx^2) (4-neighbour sum - 4 phi_t) + dt C_t phi_t
# with C the seven-term series in x and t of Appendix B, phi_0 =
# sin(pi x) sin(pi y), target_t = phi_0 + (1/4) sin(pi t) sin(2 pi x) sin(pi y)
# and L = (1/T) sum_{t=1..T} |phi_t - target_t|^2 (time t = step * dt).
#
# The estimator of Section 5 samples dL/dphi_t and the diagonal
# dphi_{t+1}/dC_t = dt diag(phi_t) with the matrix P of phi_t, so that only the
# sampled entries of phi_t are kept; the Jacobians dphi_{j+1}/dphi_j =
# M + dt diag(C_j) are known without phi, and C is recomputed from theta and t.
# Reading (the paper does not say how entries are drawn): every interior entry
# of phi_t is kept independently with probability p and scaled by 1/p; entry
# c = (i-1)(n-1) + (j-1) of step t takes the key of flat index c with
# step = t in the element_keys addressing and is kept iff key < round(p 2^32).
# Pins (tests/test_oracle_pde.py): the eigenfunction decay closed form, the
# stability number of Appendix B, p = 1 against finite differences and torch
# autograd, unbiasedness over seeds.
# ----------------------------------------------------------------------------
def pde_basis(n, t):
    """[7, n+1]: the seven functions of (x, t) whose theta-weighted sum is C."""
    x = np.arange(n + 1, dtype=np.float64) / n
    s, c = math.sin(math.pi * t), math.cos(math.pi * t)
    s2, c2 = np.sin(2 * np.pi * x), np.cos(2 * np.pi * x)
    one = np.ones(n + 1)
    return np.stack([one, s * one, c * one, s2 * s, s2 * c, c2 * s, c2 * c])


def pde_phi0(n):
    x = np.arange(n + 1, dtype=np.float64) / n
    phi = np.outer(np.sin(np.pi * x), np.sin(np.pi * x))
    phi[0, :] = phi[n, :] = 0.0
    phi[:, 0] = phi[:, n] = 0.0
    return phi


def pde_target(n, t, phi0):
    x = np.arange(n + 1, dtype=np.float64) / n
    tg = phi0 + 0.25 * math.sin(math.pi * t) * np.outer(np.sin(2 * np.pi * x), np.sin(np.pi * x))
    tg[0, :] = tg[n, :] = 0.0
    tg[:, 0] = tg[:, n] = 0.0
    return tg


def _pde_apply(phi, r, dtC):
    """(M + dt diag(C)) phi on the interior; the boundary stays zero.  dtC [n+1] varies along x (axis 0)."""
    out = np.zeros_like(phi)
    out[1:-1, 1:-1] = (phi[1:-1, 1:-1]
                       + r * (phi[2:, 1:-1] + phi[:-2, 1:-1] + phi[1:-1, 2:] + phi[1:-1, :-2] - 4.0 * phi[1:-1, 1:-1])
                       + dtC[1:-1, None] * phi[1:-1, 1:-1])
    return out


def pde_forward(theta, n, steps, D=0.25, dt=1.0 / 4096):
    """All states phi_0 .. phi_steps [steps+1, n+1, n+1] and the loss."""
    theta = np.asarray(theta, dtype=np.float64)
    r = D * dt * n * n
    phi0 = pde_phi0(n)
    phis = np.zeros((steps + 1, n + 1, n + 1))
    phis[0] = phi0
    loss = 0.0
    for t in range(steps):
        C = theta @ pde_basis(n, t * dt)
        phis[t + 1] = _pde_apply(phis[t], r, dt * C)
        loss += float(((phis[t + 1] - pde_target(n, (t + 1) * dt, phi0)) ** 2).sum())
    return phis, loss / steps


def pde_keep_mask(n, t, p, seed, stream_id):
    """[n+1, n+1] bool: kept entries of phi_t (interior only)."""
    m = n - 1
    keys = element_keys(seed, stream_id, t, 0, m * m).astype(np.uint64)
    thr = np.uint64(int(round(p * 4294967296.0)))
    mask = np.zeros((n + 1, n + 1), dtype=bool)
    mask[1:-1, 1:-1] = (keys < thr).reshape(m, m)
    return mask


def pde_rad_gradient(theta, n, steps, p, seed, stream_id=0, D=0.25, dt=1.0 / 4096):
    """(loss, dL/dtheta estimate [7], number of stored entries).  p = 1 keeps everything: the exact gradient."""
    theta = np.asarray(theta, dtype=np.float64)
    r = D * dt * n * n
    phis, loss = pde_forward(theta, n, steps, D, dt)
    phi0 = phis[0]
    masks = [pde_keep_mask(n, t, p, seed, stream_id) for t in range(steps + 1)]
    stored = int(sum(m.sum() for m in masks))
    lam = np.zeros((n + 1, n + 1))
    g = np.zeros(7)
    for t in range(steps, 0, -1):
        lam = lam + (2.0 / steps) * np.where(masks[t], (phis[t] - pde_target(n, t * dt, phi0)) / p, 0.0)
        basis = pde_basis(n, (t - 1) * dt)
        w = dt * np.where(masks[t - 1], phis[t - 1] / p, 0.0) * lam          # dL/dC_{t-1}, entry by entry
        g += basis @ w.sum(axis=1)
        lam = _pde_apply(lam, r, dt * (theta @ basis))                       # M + dt diag(C) is symmetric
    return loss, g, stored


# ----------------------------------------------------------------------------
# Reverse-mode AD with path sampling on a general computational graph
# (Appendix C, Algorithm 1).  The graph is given linearised: vertices numbered
# in topological order, vertex v with successors succ[succ_ptr[v] :
# succ_ptr[v+1]] and the partial derivatives d succ / d v on those edges.  In
# topological order, every vertex that an input vertex reaches through sampled
# edges (the inputs themselves to begin with) draws k of its d_v outgoing edges
# uniformly with replacement and adds (d_v / k) * partial to Q of each drawn
# edge; vertices no sampled edge leads to are skipped.  Back-propagation from y
# with Q as the edge partials gives the estimate: v^ = sum_e Q(e) succ(e)^,
# y^ = 1.  Draw s of vertex v takes the key of flat index v k + s and maps it
# to edge floor(key d_v / 2^32) of v (the mapping of the with-replacement
# schemes).  `draws`, if given, replaces the keys (tests enumerate outcomes).
# Pins (tests/test_oracle_paths.py): the expectation over every outcome of the
# draws on small graphs equals the exact derivative; chains are exact; the
# mean over seeds on random layered graphs; unreached vertices stay zero.
# ----------------------------------------------------------------------------
def graph_exact_adjoints(succ_ptr, succ, partial, y):
    n = len(succ_ptr) - 1
    adj = np.zeros(n)
    adj[y] = 1.0
    for v in range(n - 1, -1, -1):
        if v == y:
            continue
        e0, e1 = succ_ptr[v], succ_ptr[v + 1]
        adj[v] = float(np.dot(partial[e0:e1], adj[succ[e0:e1]]))
    return adj


def path_sample_adjoints(succ_ptr, succ, partial, y, inputs, k, seed, stream_id=0, draws=None):
    """Estimates v^ of dy/dv for every vertex (zero where the vertex was skipped); the gradient is v^ at the
    input vertices.  draws: optional {vertex: [k edge numbers in 0 .. d_v - 1]}."""
    succ_ptr = np.asarray(succ_ptr, dtype=np.int64)
    succ = np.asarray(succ, dtype=np.int64)
    partial = np.asarray(partial, dtype=np.float64)
    n = len(succ_ptr) - 1
    reached = np.zeros(n, dtype=bool)
    reached[np.asarray(inputs, dtype=np.int64)] = True
    picks = {}
    for v in range(n):
        d = int(succ_ptr[v + 1] - succ_ptr[v])
        if not reached[v] or d == 0:
            continue
        if draws is not None:
            idx = np.asarray(draws[v], dtype=np.int64)
        else:
            keys = element_keys(seed, stream_id, 0, v * k, k).astype(np.uint64)
            idx = ((keys * np.uint64(d)) >> np.uint64(32)).astype(np.int64)
        picks[v] = succ_ptr[v] + idx
        reached[succ[picks[v]]] = True
    adj = np.zeros(n)
    if reached[y]:
        adj[y] = 1.0
    for v in range(n - 1, -1, -1):
        if v == y or v not in picks:
            continue
        d = int(succ_ptr[v + 1] - succ_ptr[v])
        e = picks[v]
        adj[v] = (d / k) * float(np.sum(partial[e] * adj[succ[e]]))      # a drawn edge counts once per draw
    return adj, reached


# ----------------------------------------------------------------------------
# Byte accounting, in the paper's convention (Appendix A, "Calculation of
# memory saved from RAD"): 32-bit values for the stored (sampled) inputs,
# ceil(p d) of them per input, one bit per un-reduced ReLU entry, the softmax
# input unsampled, nothing for pooling and biases; indices are not counted.
# ----------------------------------------------------------------------------
def paper_bytes_per_example(sampled_dims, logits, relu_entries, p):
    if p >= 1.0:
        return 4.0 * (sum(sampled_dims) + logits)
    vals = sum(fixed_k(p, d) for d in sampled_dims) + logits
    return 4.0 * vals + relu_entries / 8.0


def paper_total_megabytes(n_params, batch, sampled_dims, logits, relu_entries, p):
    """Table 1: weights plus batch * per-example bytes, in 10^6-byte MB."""
    return (4.0 * n_params + batch * paper_bytes_per_example(
        sampled_dims, logits, relu_entries, p)) / 1e6

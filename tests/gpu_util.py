"""Helpers shared by the GPU parity tests: device buffers via torch (plumbing
only), bit unpacking, error norms."""
import numpy as np
import torch

from paper_2007_10412_amd import binding as B

TOL = {B.RAD_F32: 1e-4, B.RAD_BF16: 2e-2}   # relative Frobenius error on gradients (the tolerance the benchmark spec states)


def dev(a, dtype=B.RAD_F32):
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if dtype == B.RAD_BF16 and t.dtype == torch.float32:
        t = t.to(torch.bfloat16)
    return t.contiguous()


def host(t):
    return t.detach().to(torch.float32).cpu().numpy() if t.dtype == torch.bfloat16 else t.detach().cpu().numpy()


def empty(shape, dtype=B.RAD_F32):
    return torch.empty(shape, device="cuda", dtype=torch.bfloat16 if dtype == B.RAD_BF16 else torch.float32)


def unpack_bits(words, n):
    """[rows, ceil(n/32)] uint32 -> bool [rows, n]"""
    w = np.asarray(words, dtype=np.uint32)
    bits = (w[:, :, None] >> np.arange(32, dtype=np.uint32)[None, None, :]) & 1
    return bits.reshape(w.shape[0], -1)[:, :n].astype(bool)


def pack_bits(b):
    rows, n = b.shape
    nw = (n + 31) // 32
    pad = np.zeros((rows, nw * 32), dtype=np.uint32)
    pad[:, :n] = b
    return (pad.reshape(rows, nw, 32) << np.arange(32, dtype=np.uint32)[None, None, :]).sum(axis=2).astype(np.uint32)


def rel_err(got, want):
    want = np.asarray(want, dtype=np.float64)
    got = np.asarray(got, dtype=np.float64)
    den = np.linalg.norm(want)
    return np.linalg.norm(got - want) / (den if den > 0 else 1.0)


def assert_bits_match(bits_gpu, h_oracle, tag=""):
    """ReLU bits must agree except where the oracle's pre-activation is within rounding of zero."""
    want = h_oracle > 0
    diff = bits_gpu != want
    if diff.any():
        rms = np.sqrt(np.mean(h_oracle**2))
        assert np.all(np.abs(h_oracle[diff]) <= 1e-5 * rms), tag + ": ReLU bit differs away from zero"
        assert diff.mean() < 0.01, tag
    return int(diff.sum())

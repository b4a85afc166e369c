"""Helpers for the GPU parity tests (marshalling between numpy and torch device tensors)."""
import numpy as np
import torch


def dev(a):
    """numpy array -> CUDA tensor with the same bytes (uint16 travels as int16)."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    if a.dtype == np.uint32:
        return torch.from_numpy(a.view(np.int32)).cuda()
    return torch.from_numpy(a).cuda()


def host(t):
    """CUDA code tensor -> numpy (uint16 / uint8)."""
    t = t.cpu()
    if t.dtype == torch.uint16:
        return t.view(torch.int16).numpy().view(np.uint16)
    if t.dtype == torch.int16:
        return t.numpy().view(np.uint16)
    return t.numpy()


def first_mismatch(got, want):
    idx = np.flatnonzero(got != want)
    if idx.size == 0:
        return None
    i = int(idx[0])
    return "%d mismatches, first at %d: got 0x%x want 0x%x" % (idx.size, i, int(got[i]), int(want[i]))


def assert_stats_close(got, want, rel=1e-6):
    """count exact; sums within rel relative, sum e with an absolute floor of rel (its mean is
    near zero for unbiased variants); non-finite entries must agree in kind."""
    got = np.asarray(got, dtype=np.float64).reshape(-1, 4)
    want = np.asarray(want, dtype=np.float64).reshape(-1, 4)
    assert np.array_equal(got[:, 0], want[:, 0]), "counts differ"
    for col in (1, 2, 3):
        g, w = got[:, col], want[:, col]
        assert np.array_equal(np.isnan(g), np.isnan(w)), "NaN pattern differs in column %d" % col
        fin = np.isfinite(w)
        assert np.array_equal(g[~fin & ~np.isnan(w)], w[~fin & ~np.isnan(w)]), "infinities differ"
        tol = rel * np.maximum(np.abs(w[fin]), 1.0 if col == 2 else 0.0)
        bad = np.abs(g[fin] - w[fin]) > tol
        assert not bad.any(), "column %d: %d bins off, worst %g" % (
            col, bad.sum(), np.max(np.abs(g[fin] - w[fin]) / np.maximum(np.abs(w[fin]), 1e-300)))

"""Comparators shared by the GPU parity tests.

Tolerances: attention outputs and scores agree with
the fp64 oracle within 1e-5 relative error in fp32 and 2e-2 in bf16; the elementwise rule is
|x - y| <= rtol * |y| + atol with atol = rtol * RMS(y).  Top-k index sets must match exactly
except for candidates whose oracle score lies within that tolerance of the k-th score.
"""
import numpy as np
import torch

RTOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


def to_np(t):
    return t.detach().float().cpu().numpy() if t.dtype in (torch.bfloat16, torch.float16) \
        else t.detach().cpu().numpy()


def assert_close(got, want, rtol, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    atol = rtol * float(np.sqrt(np.mean(want ** 2))) if want.size else 0.0
    err = np.abs(got - want)
    bound = rtol * np.abs(want) + atol
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())}/{bad.size} outside tolerance; worst at {i}: "
                             f"got {got[i]!r} want {want[i]!r} err {err[i]:.3e} bound {bound[i]:.3e}")


def assert_selection_within_band(got_idx, oracle_score, keep, rtol, what="", forced=()):
    """got_idx: selected indices (ascending expected); oracle_score: fp64 scores of all candidates.

    Returns the number of in-band substitutions relative to the oracle's exact choice.
    """
    got = np.asarray(got_idx, dtype=np.int64)
    s = np.asarray(oracle_score, dtype=np.float64).copy()
    n = s.shape[0]
    assert got.shape == (keep,), (what, got.shape, keep)
    assert np.all(np.diff(got) > 0), f"{what}: indices not strictly ascending"
    assert got.min() >= 0 and got.max() < n, f"{what}: index out of range"
    forced = np.asarray(sorted(forced), dtype=np.int64)
    if forced.size:
        assert np.isin(forced, got).all(), f"{what}: a protected slot was dropped"
        s[forced] = np.inf
    order = np.lexsort((np.arange(n), -s))          # value descending, index ascending
    exact = np.sort(order[:keep])
    tau = s[order[keep - 1]]
    if not np.isfinite(tau):
        eps = 0.0
    else:
        eps = rtol * abs(tau) + rtol * float(np.sqrt(np.mean(np.where(np.isfinite(s), s, 0.0) ** 2)))
    chosen = np.zeros(n, bool)
    chosen[got] = True
    must = s > tau + eps
    never = s < tau - eps
    assert chosen[must].all(), f"{what}: {int((~chosen[must]).sum())} clear winners missing"
    assert not chosen[never].any(), f"{what}: {int(chosen[never].sum())} clear losers selected"
    return int(np.setdiff1d(got, exact).size)


def numpy_union(topk, N, radius, n_head, n_tail):
    """Plain numpy statement of the union with dilation (independent of the oracle and the GPU)."""
    t = np.asarray(topk, dtype=np.int64).reshape(-1, 1) + np.arange(-radius, radius + 1)[None, :]
    t = t[(t >= 0) & (t < N)]
    extra = np.concatenate([np.arange(min(n_head, N)), np.arange(max(N - n_tail, 0), N)])
    return np.unique(np.concatenate([t.ravel(), extra])).astype(np.int32)

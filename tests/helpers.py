"""Comparators shared by the GPU parity tests.

Tolerances: attention outputs and scores agree with
the fp64 oracle within 1e-5 relative error in fp32 and 2e-2 in bf16; the elementwise rule is
|x - y| <= rtol * |y| + atol with atol = rtol * RMS(y); eviction scores take the floor per head
from the typical candidates only (assert_scores_close).  Top-k index sets must match exactly
except for candidates whose oracle score lies within rtol * |k-th score| of the k-th score.
"""
import numpy as np
import torch

RTOL = {torch.float32: 1e-5, torch.bfloat16: 2e-2}


def to_np(t):
    return t.detach().float().cpu().numpy() if t.dtype in (torch.bfloat16, torch.float16) \
        else t.detach().cpu().numpy()


def _raise_worst(what, got, want, err, bound):
    bad = err > bound
    i = np.unravel_index(np.argmax(err - bound), err.shape)
    raise AssertionError(f"{what}: {int(bad.sum())}/{bad.size} outside tolerance; worst at {i}: "
                         f"got {got[i]!r} want {want[i]!r} err {err[i]:.3e} bound {bound[i]:.3e}")


def assert_close(got, want, rtol, what="", row_floor=False):
    """|got - want| <= rtol * |want| + rtol * RMS(want), RMS over the whole tensor.

    row_floor (attention outputs [.., rows, d]): the floor of a row is the larger of the tensor's
    RMS and the row's own RMS.  The probabilities fed to the P.V product are rounded to bf16
    (relative error up to 2^-8 each), so element c of a row carries an error of up to
    2^-8 * sum_j p_j |v_jc|: a row whose attention sits on a few keys is larger than the average
    row AND carries a proportionally larger error, also in elements where the contributions of
    those keys cancel; against the row's own scale that error stays below 2^-8 * max|v| / RMS(v)."""
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    atol = rtol * float(np.sqrt(np.mean(want ** 2))) if want.size else 0.0
    if row_floor and want.size:
        atol = np.maximum(atol, rtol * np.sqrt(np.mean(want ** 2, axis=-1, keepdims=True)))
    err = np.abs(got - want)
    bound = rtol * np.abs(want) + atol
    if (err > bound).any():
        _raise_worst(what, got, want, err, bound)


def robust_scale(row):
    """RMS of the entries of `row` at or below the 99th percentile of |row|: the size of a typical
    entry, which a handful of huge ones (attention sinks, needles) do not move."""
    a = np.abs(np.asarray(row, dtype=np.float64))
    if a.size == 0:
        return 0.0
    body = a[a <= np.percentile(a, 99.0)]
    return float(np.sqrt(np.mean(body ** 2))) if body.size else 0.0


def assert_scores_close(got, want, rtol, what=""):
    """Eviction scores [rows][candidates]: |got - want| <= rtol * |want| + rtol * robust_scale(row).

    The absolute floor is taken per row from the typical candidates only, so that a few dominant
    keys (whose scores can be thousands of times the median) cannot widen it until an ordinary
    key's score could be anything.  The whole-tensor rule of assert_close is implied (its floor is
    never smaller)."""
    got = np.atleast_2d(np.asarray(got, dtype=np.float64))
    want = np.atleast_2d(np.asarray(want, dtype=np.float64))
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite values"
    floor = np.array([rtol * robust_scale(r) for r in want.reshape(-1, want.shape[-1])])
    floor = floor.reshape(want.shape[:-1] + (1,))
    err = np.abs(got - want)
    bound = rtol * np.abs(want) + floor
    if (err > bound).any():
        _raise_worst(what, got, want, err, bound)


# Filled by assert_selection_within_band for the caller to report: candidates inside the band,
# share of candidates the band decides (must or never), substitutions against the oracle's exact
# choice, and how many of the GPU's choices would violate the tight band rtol = 1e-5.
LAST_BAND = {}


def band_sets(s, keep, rtol):
    """Threshold tau = keep-th largest score (ties to the lowest index) and the band
    eps = rtol * |tau| around it: returns (exact choice ascending, must, never) as index / masks."""
    n = s.shape[0]
    order = np.lexsort((np.arange(n), -s))          # value descending, index ascending
    exact = np.sort(order[:keep])
    tau = s[order[keep - 1]]
    eps = rtol * abs(tau) if np.isfinite(tau) else 0.0
    return exact, s > tau + eps, s < tau - eps


def assert_selection_within_band(got_idx, oracle_score, keep, rtol, what="", forced=()):
    """got_idx: selected indices (ascending expected); oracle_score: fp64 scores of all candidates.

    Every candidate whose oracle score exceeds tau + eps must be selected, none below tau - eps may
    be, eps = rtol * |tau|; inside the band any choice is accepted.  Returns the number of in-band
    substitutions relative to the oracle's exact choice; LAST_BAND holds the other statistics.
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
    exact, must, never = band_sets(s, keep, rtol)
    chosen = np.zeros(n, bool)
    chosen[got] = True
    assert chosen[must].all(), f"{what}: {int((~chosen[must]).sum())} clear winners missing"
    assert not chosen[never].any(), f"{what}: {int(chosen[never].sum())} clear losers selected"
    subs = int(np.setdiff1d(got, exact).size)
    _, must_t, never_t = band_sets(s, keep, 1e-5)
    LAST_BAND.clear()
    LAST_BAND.update(in_band=int(n - must.sum() - never.sum()),
                     decided=float((must.sum() + never.sum()) / n), subs=subs,
                     tight_violations=int((~chosen[must_t]).sum() + chosen[never_t].sum()))
    return subs


class BandTally:
    """Sums LAST_BAND over the selections of a test, for one printed line."""

    def __init__(self):
        self.rows = self.subs = self.in_band = self.tight = 0
        self.decided_min = 1.0

    def add(self):
        self.rows += 1
        self.subs += LAST_BAND["subs"]
        self.in_band += LAST_BAND["in_band"]
        self.tight += LAST_BAND["tight_violations"]
        self.decided_min = min(self.decided_min, LAST_BAND["decided"])

    def __str__(self):
        return (f"{self.rows} selections: {self.subs} in-band substitutions, {self.in_band} candidates "
                f"in band, band decides >= {100 * self.decided_min:.1f} % of candidates, "
                f"{self.tight} choices outside the tight band (rtol 1e-5)")


def numpy_union(topk, N, radius, n_head, n_tail):
    """Plain numpy statement of the union with dilation (independent of the oracle and the GPU)."""
    t = np.asarray(topk, dtype=np.int64).reshape(-1, 1) + np.arange(-radius, radius + 1)[None, :]
    t = t[(t >= 0) & (t < N)]
    extra = np.concatenate([np.arange(min(n_head, N)), np.arange(max(N - n_tail, 0), N)])
    return np.unique(np.concatenate([t.ravel(), extra])).astype(np.int32)


def oracle_kv_heads_dense(q, K, V, M, scale, kv_heads, threads=None):
    """The oracle's attend_score for a subset of KV heads, with the query rows spread over Python
    threads (the C routine parallelises over KV heads only, which leaves a one- or two-head check
    on a single core).  Each thread asks oracle.attend_rows for its rows of the group and for the
    attention mass those rows alone contribute; the partial masses are added in fp64.

    q [Hq,Ct,d], K, V [Hkv,cap,d] float32 arrays.  Returns (out [len(kv_heads)*G, Ct, d],
    lse [len(kv_heads)*G, Ct], score [len(kv_heads), M+Ct]) for the whole chunk as observers."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    import oracle
    Hq, Ct, d = q.shape
    Hkv = K.shape[0]
    G = Hq // Hkv
    kv_heads = list(kv_heads)
    nh = len(kv_heads) * G
    qs = np.ascontiguousarray(np.concatenate([q[g * G:(g + 1) * G] for g in kv_heads]), dtype=np.float32)
    Ks = np.ascontiguousarray(K[kv_heads], dtype=np.float32)
    Vs = np.ascontiguousarray(V[kv_heads], dtype=np.float32)
    n = M + Ct
    threads = threads or min(16, len(os.sched_getaffinity(0)))
    hh, ii = np.meshgrid(np.arange(nh, dtype=np.int32), np.arange(Ct, dtype=np.int32), indexing="ij")
    hh, ii = hh.ravel(), ii.ravel()
    order = np.argsort(-ii, kind="stable")             # long rows first, dealt round-robin
    parts = [order[t::threads] for t in range(threads)]

    def work(sel):
        oracle.set_num_threads(1)
        return oracle.attend_rows(qs, Ks, Vs, M, scale, hh[sel], ii[sel], want_score=True)

    out = np.zeros((nh, Ct, d), np.float64)
    lse = np.zeros((nh, Ct), np.float64)
    score = np.zeros((len(kv_heads), n), np.float64)
    with ThreadPoolExecutor(max_workers=threads) as ex:
        for sel, (o, l, s) in zip(parts, ex.map(work, parts)):
            out[hh[sel], ii[sel]] = o
            lse[hh[sel], ii[sel]] = l
            score += s[:, :n]
    return out, lse, score


def build_store_gpu(raw, head_dim=128):
    """The embedding store the GPU path makes of raw head states [N, D] (device tensor): one
    reform_embed_save_selected call normalises the D/head_dim segments of every row."""
    from paper_2506_01215_amd import binding
    N, D = raw.shape
    store = torch.empty_like(raw)
    binding.reform_embed_save_selected(raw.view(N, D // head_dim, head_dim).permute(1, 0, 2), store, 0, 0)
    return store


def build_store_oracle(raw, head_dim=128, block=65536):
    """The same store by the oracle's own routine (fp64, then rounded to the storage type), from
    the same raw head states; returns a host tensor of raw's dtype."""
    import oracle
    N, D = raw.shape
    out = torch.empty((N, D), dtype=raw.dtype)
    for r0 in range(0, N, block):
        r1 = min(N, r0 + block)
        src = raw[r0:r1].float().cpu().numpy()
        emb = np.zeros((r1 - r0, D), np.float64)
        for h in range(D // head_dim):
            oracle.embed_segment(src[:, h * head_dim:(h + 1) * head_dim], emb, h * head_dim)
        out[r0:r1] = torch.from_numpy(emb).to(raw.dtype)
    return out


def stores_for(cfg, emb, qry):
    """(GPU-side emb, qry on the device; oracle-side emb, qry on the host) for a gather workload:
    the same tensors for kind "iid", each side's own embedding construction for "head_states"."""
    dev = "cuda:0"
    if cfg.kind == "head_states":
        return (build_store_gpu(emb.to(dev)), build_store_gpu(qry.to(dev)),
                build_store_oracle(emb), build_store_oracle(qry))
    return emb.to(dev), qry.to(dev), emb.cpu(), qry.cpu()

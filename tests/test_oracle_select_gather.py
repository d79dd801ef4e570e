"""Pins for the CPU oracle's retention, compaction and gather (no GPU needed).

Independent references: Python's exhaustive `sorted` with an explicit
(value, index) key, python sets for the union, numpy/torch library routines for
the cosine and for max-pooling, and the paper's identity that cosine over the
concatenation of L2-normalised head states equals the mean of the per-head
cosines (Sec. 3.2, equation for e_comb and the sentence after it).
"""
import numpy as np
import pytest
import torch

import oracle


def exhaustive_topk(x, keep, forced=()):
    key = [(-(np.inf if j in forced else x[j]), j) for j in range(len(x))]
    order = [j for _, j in sorted(key)]
    return sorted(order[:keep])


@pytest.mark.parametrize("n,B,seed", [(1, 1, 0), (10, 3, 1), (64, 32, 2), (257, 100, 3), (50, 50, 4)])
def test_topk_matches_exhaustive_sort(n, B, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal(n)
    assert list(oracle.topk_lowest_index(x, B)) == exhaustive_topk(x, B)


def test_ties_go_to_lowest_index():
    x = np.array([1.0, 3.0, 2.0, 3.0, 2.0, 2.0, 0.5, 2.0])
    assert list(oracle.topk_lowest_index(x, 3)) == [1, 2, 3]          # the first of the four 2.0s
    assert list(oracle.topk_lowest_index(x, 5)) == [1, 2, 3, 4, 5]
    assert list(oracle.topk_lowest_index(np.zeros(9), 4)) == [0, 1, 2, 3]
    rng = np.random.default_rng(11)
    x = rng.integers(0, 5, size=200).astype(np.float64)              # heavy ties
    for keep in (1, 17, 100, 199):
        assert list(oracle.topk_lowest_index(x, keep)) == exhaustive_topk(x, keep)


def test_evict_select_invariants_and_forced_slots():
    rng = np.random.default_rng(12)
    n, B = 300, 64
    s = rng.random(n)
    kept = oracle.evict_select(s, n, B)
    assert len(kept) == B and np.all(np.diff(kept) > 0)
    evicted = np.setdiff1d(np.arange(n), kept)
    assert s[kept].min() >= s[evicted].max()
    # n <= B keeps everything
    assert list(oracle.evict_select(s, 40, 64)) == list(range(40))
    # sinks and recents are kept regardless of score and count inside B
    s2 = s.copy()
    s2[:4] = -1.0
    s2[-8:] = -1.0
    kept = oracle.evict_select(s2, n, B, n_sink=4, n_recent=8)
    forced = set(range(4)) | set(range(n - 8, n))
    assert len(kept) == B and forced <= set(kept.tolist())
    assert list(kept) == exhaustive_topk(s2, B, forced)
    with pytest.raises(ValueError):
        oracle.evict_select(s, n, 8, n_sink=5, n_recent=5)


def test_compaction_is_order_preserving_row_gather():
    rng = np.random.default_rng(13)
    Hkv, cap, d, n, B = 3, 40, 5, 37, 16
    k = rng.standard_normal((Hkv, cap, d)).astype(np.float32)
    v = rng.standard_normal((Hkv, cap, d)).astype(np.float32)
    s = rng.random((Hkv, cap))
    pos = np.tile(np.arange(cap, dtype=np.int32) + 1000, (Hkv, 1))
    k2, v2, s2, p2, kept = oracle.evict_compact(k, v, s, pos, n, B)
    for g in range(Hkv):
        idx = exhaustive_topk(s[g, :n], B)
        assert list(kept[g]) == idx
        np.testing.assert_array_equal(k2[g, :B], k[g, idx])
        np.testing.assert_array_equal(v2[g, :B], v[g, idx])
        np.testing.assert_array_equal(s2[g, :B], s[g, idx])
        np.testing.assert_array_equal(p2[g, :B], pos[g, idx])
        assert np.all(np.diff(p2[g, :B]) > 0)            # original order survives
        np.testing.assert_array_equal(k2[g, B:], k[g, B:])  # rows past the new length untouched


def test_cosine_matches_library_and_clamp():
    rng = np.random.default_rng(14)
    emb = rng.standard_normal((50, 24)).astype(np.float32)
    qry = rng.standard_normal((3, 24)).astype(np.float32)
    emb[7] = 0.0                                           # zero row: clamp, result 0
    sim = oracle.cosine(emb, qry, eps=1e-8)
    ref = torch.nn.functional.cosine_similarity(
        torch.from_numpy(qry).double()[:, None, :], torch.from_numpy(emb).double()[None, :, :],
        dim=-1, eps=1e-8).numpy()
    mask = np.arange(50) != 7
    np.testing.assert_allclose(sim[:, mask], ref[:, mask], rtol=1e-12, atol=1e-14)
    assert np.all(sim[:, 7] == 0)
    assert np.all(np.abs(sim) <= 1 + 1e-12)
    # self-similarity is 1, negation is -1
    sim2 = oracle.cosine(emb[:5], emb[:5])
    np.testing.assert_allclose(np.diag(sim2), 1.0, rtol=1e-12)
    np.testing.assert_allclose(oracle.cosine(-emb[:5], emb[:5]).diagonal(), -1.0, rtol=1e-12)


def test_concat_of_normalised_heads_is_mean_of_per_head_cosines():
    rng = np.random.default_rng(15)
    N, heads, hd = 40, 4, 16
    e = rng.standard_normal((N, heads, hd)) * rng.uniform(0.1, 10, size=(N, heads, 1))
    u = rng.standard_normal((2, heads, hd)) * rng.uniform(0.1, 10, size=(2, heads, 1))
    en = e / np.linalg.norm(e, axis=-1, keepdims=True)
    un = u / np.linalg.norm(u, axis=-1, keepdims=True)
    whole = oracle.cosine(en.reshape(N, -1), un.reshape(2, -1))
    per_head = np.stack([oracle.cosine(e[:, h], u[:, h]) for h in range(heads)]).mean(axis=0)
    # float32 storage of the normalised vectors limits the agreement, not the oracle
    np.testing.assert_allclose(whole, per_head, atol=3e-7)


def test_gather_reductions():
    rng = np.random.default_rng(16)
    emb = rng.standard_normal((120, 12)).astype(np.float32)
    qry = rng.standard_normal((3, 12)).astype(np.float32)
    sim, topk, uni = oracle.gather(emb, qry, k=120)
    assert all(list(topk[q]) == list(range(120)) for q in range(3))      # k = N: everything
    sim, topk, uni = oracle.gather(emb, qry[:1], k=10)
    assert list(uni) == list(topk[0])                                      # nq = 1, r = 0
    assert list(topk[0]) == exhaustive_topk(sim[0], 10)
    sim, topk, uni = oracle.gather(emb, qry, k=9, radius=2, n_head=3, n_tail=4)
    want = set(range(3)) | set(range(116, 120))
    for q in range(3):
        assert list(topk[q]) == exhaustive_topk(sim[q], 9)
        for t in topk[q]:
            want |= {t + dlt for dlt in range(-2, 3) if 0 <= t + dlt < 120}
    assert list(uni) == sorted(want)
    assert np.all(np.diff(uni) > 0) and uni.min() >= 0 and uni.max() < 120


def test_dilation_is_maxpool_in_threshold_form():
    """{t : maxpool_{2r+1}(s)_t >= tau} == dilate_r({t : s_t >= tau}) (Sec. 3.3 pooling motive)."""
    rng = np.random.default_rng(17)
    N, r, k = 300, 8, 12
    s = rng.standard_normal(N)
    top = oracle.topk_lowest_index(s, k)
    tau = s[top].min()
    pooled = torch.nn.functional.max_pool1d(torch.from_numpy(s)[None, None], 2 * r + 1, stride=1,
                                            padding=r)[0, 0].numpy()
    want = np.nonzero(pooled >= tau)[0]
    got = oracle.union_dilate(top[None, :], N, radius=r)
    np.testing.assert_array_equal(got, want)


# ---- the paper's own post-processing (Sec. 3.3): max over query tokens, window max-pool, top budget

def brute_pool(sim, window):
    nq, N = sim.shape
    h = (window - 1) // 2
    s = [max(sim[q][t] for q in range(nq)) for t in range(N)]
    return np.array([max(s[max(0, t - h):min(N, t + h + 1)]) for t in range(N)])


@pytest.mark.parametrize("nq,N,window", [(1, 1, 1), (3, 40, 5), (4, 300, 129), (2, 64, 17), (5, 130, 129), (1, 10, 129)])
def test_pool_scores_matches_brute_force_and_library_filters(nq, N, window):
    from scipy.ndimage import maximum_filter1d
    rng = np.random.default_rng(40 + N)
    sim = rng.standard_normal((nq, N))
    got = oracle.pool_scores(sim, window)
    np.testing.assert_array_equal(got, brute_pool(sim, window))
    lib = maximum_filter1d(sim.max(axis=0), size=window, mode="constant", cval=-np.inf)
    np.testing.assert_array_equal(got, lib)
    tp = torch.nn.functional.max_pool1d(torch.from_numpy(sim.max(axis=0))[None, None], window, stride=1,
                                        padding=window // 2)[0, 0].numpy()   # pads with -inf
    np.testing.assert_array_equal(got, tp)


def test_pool_scores_special_cases():
    rng = np.random.default_rng(41)
    sim = rng.standard_normal((6, 200))
    np.testing.assert_array_equal(oracle.pool_scores(sim, 1), sim.max(axis=0))      # window 1: only the query max
    np.testing.assert_array_equal(oracle.pool_scores(sim[:1], 1), sim[0])           # one query, window 1: identity
    np.testing.assert_array_equal(oracle.pool_scores(sim, 401), np.full(200, sim.max()))   # window covers everything
    spike = np.full((1, 50), -1.0)
    spike[0, 20] = 2.0
    want = np.full(50, -1.0)
    want[18:23] = 2.0                                                               # a spike becomes a plateau of `window`
    np.testing.assert_array_equal(oracle.pool_scores(spike, 5), want)
    with pytest.raises(ValueError):
        oracle.pool_scores(sim, 4)                                                  # even windows have no centre


def test_gather_pooled_end_to_end_small():
    """cosine -> pooled score -> budget selection with forced ends, against python sets/sorts."""
    rng = np.random.default_rng(42)
    N, D, nq, budget, window = 500, 16, 3, 60, 9
    emb = rng.standard_normal((N, D)).astype(np.float32)
    qry = rng.standard_normal((nq, D)).astype(np.float32)
    sim, pooled, sel = oracle.gather_pooled(emb, qry, budget, window, n_head=8, n_tail=8)
    np.testing.assert_array_equal(pooled, brute_pool(sim, window))
    forced = set(range(8)) | set(range(N - 8, N))
    assert list(sel) == exhaustive_topk(pooled, budget, forced)
    assert len(sel) == budget and forced <= set(sel.tolist())
    # plateaus: equal pooled scores are taken from the lowest index on
    free = [t for t in sel if t not in forced]
    thr = min(pooled[t] for t in free)
    below = [t for t in range(N) if t not in forced and t not in set(sel.tolist())]
    assert all(pooled[t] <= thr for t in below)
    ties_out = [t for t in below if pooled[t] == thr]
    ties_in = [t for t in free if pooled[t] == thr]
    if ties_out and ties_in:
        assert max(ties_in) < min(ties_out)


def test_forced_slots_filling_the_budget_ignore_the_scores():
    """n_sink + n_recent = B is the StreamingLLM rule: first and latest tokens, whatever the scores."""
    rng = np.random.default_rng(50)
    s = rng.standard_normal(100)
    kept = oracle.evict_select(s, 100, 20, n_sink=4, n_recent=16)
    assert list(kept) == list(range(4)) + list(range(84, 100))


# ---- embedding construction (Sec. 3.2 "Combining multiple heads", Alg. 1 SaveSelected)

def test_embed_segment_unit_norm_placement_and_strides():
    rng = np.random.default_rng(60)
    n, d, D = 37, 16, 64
    big = rng.standard_normal((n, 3 * d)).astype(np.float32)       # the head sits inside a wider row
    src = big[:, d:2 * d]
    emb = np.full((n, D), 7.0)
    oracle.embed_segment(src, emb, col=32)
    want = src.astype(np.float64) / np.linalg.norm(src.astype(np.float64), axis=1, keepdims=True)
    np.testing.assert_allclose(emb[:, 32:48], want, rtol=1e-14)
    np.testing.assert_allclose(np.linalg.norm(emb[:, 32:48], axis=1), 1.0, rtol=1e-14)
    assert np.all(emb[:, :32] == 7.0) and np.all(emb[:, 48:] == 7.0)      # other segments untouched
    tn = torch.nn.functional.normalize(torch.from_numpy(src).double(), dim=1).numpy()
    np.testing.assert_allclose(emb[:, 32:48], tn, rtol=1e-14)


def test_embed_segment_scale_invariance_idempotence_and_zero_rows():
    rng = np.random.default_rng(61)
    src = rng.standard_normal((9, 8)).astype(np.float32)
    a = oracle.embed_segment(src, np.zeros((9, 8)), 0)
    b = oracle.embed_segment(src * np.float32(4.0), np.zeros((9, 8)), 0)      # x4 is exact in fp32
    np.testing.assert_allclose(a, b, rtol=1e-15)
    src[3] = 0.0
    z = oracle.embed_segment(src, np.ones((9, 8)), 0)
    assert np.all(z[3] == 0.0) and np.all(np.isfinite(z))
    with pytest.raises(ValueError):
        oracle.embed_segment(src, np.zeros((9, 12)), 8)                       # segment would overrun the row


def test_combined_embedding_cosine_is_mean_of_per_head_cosines_end_to_end():
    """The sentence after the e_comb equation: a cosine search on the concatenation of the
    normalised heads equals the average of the per-head cosine scores."""
    rng = np.random.default_rng(62)
    n, d, H = 50, 12, 4
    ctx = rng.standard_normal((H, n, d)).astype(np.float32)
    qry = rng.standard_normal((H, 2, d)).astype(np.float32)
    E = np.zeros((n, H * d))
    U = np.zeros((2, H * d))
    for h in range(H):
        oracle.embed_segment(ctx[h], E, h * d)
        oracle.embed_segment(qry[h], U, h * d)
    sim = oracle.cosine(E.astype(np.float32), U.astype(np.float32))
    per_head = np.zeros((2, n))
    for h in range(H):
        a = ctx[h].astype(np.float64)
        b = qry[h].astype(np.float64)
        per_head += (b @ a.T) / (np.linalg.norm(b, axis=1)[:, None] * np.linalg.norm(a, axis=1)[None, :])
    np.testing.assert_allclose(sim, per_head / H, rtol=2e-6, atol=2e-7)      # E, U pass through float32


def test_gather_rows_is_fancy_indexing():
    rng = np.random.default_rng(70)
    table = rng.integers(0, 2 ** 16, size=(50, 24), dtype=np.uint16)       # bf16-sized raw elements
    idx = np.array([0, 3, 3, 49, 17], np.int32)
    np.testing.assert_array_equal(oracle.gather_rows(table, idx), table[idx])
    assert oracle.gather_rows(table, np.zeros(0, np.int32)).shape == (0, 24)
    with pytest.raises(ValueError):
        oracle.gather_rows(table, np.array([50], np.int32))

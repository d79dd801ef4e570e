"""Pins for the CPU oracle's chunk attention + eviction score (no GPU needed).

The paper prints no worked numeric example, so the oracle is pinned by things
that do not depend on it: a brute-force materialised softmax (numpy), torch's
CPU scaled_dot_product_attention, closed forms for uniform attention (harmonic
sums, also stored as exact rationals under tests/golden/), invariants of the
definition (total attention mass), and symmetry/limit cases.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_case(rng, Hq, Hkv, d, M, Ct, extra_cap=3):
    cap = M + Ct + extra_cap
    q = rng.standard_normal((Hq, Ct, d)).astype(np.float32)
    k = rng.standard_normal((Hkv, cap, d)).astype(np.float32)
    v = rng.standard_normal((Hkv, cap, d)).astype(np.float32)
    # rows past n are garbage the oracle must never read into a result
    k[:, M + Ct:] = np.nan
    v[:, M + Ct:] = np.nan
    return q, k, v


def brute_force(q, k, v, M, scale, W):
    """Materialise the whole masked [Ct, n] probability matrix per head (numpy, fp64)."""
    Hq, Ct, d = q.shape
    Hkv = k.shape[0]
    G = Hq // Hkv
    n = M + Ct
    W = Ct if W == 0 else W
    out = np.zeros((Hq, Ct, d))
    lse = np.zeros((Hq, Ct))
    score = np.zeros((Hkv, k.shape[1]))
    jj = np.arange(n)[None, :]
    ii = np.arange(Ct)[:, None]
    visible = jj <= (M + ii)
    for h in range(Hq):
        g = h // G
        S = (q[h].astype(np.float64) @ k[g, :n].astype(np.float64).T) * scale
        S = np.where(visible, S, -np.inf)
        E = np.exp(S - S.max(axis=1, keepdims=True))
        Z = E.sum(axis=1, keepdims=True)
        P = E / Z
        out[h] = P @ v[g, :n].astype(np.float64)
        lse[h] = S.max(axis=1) + np.log(Z[:, 0])
        score[g, :n] += P[Ct - W:].sum(axis=0)
    return out, lse, score


@pytest.mark.parametrize("Hq,Hkv,d,M,Ct,W", [
    (4, 4, 8, 0, 5, 0),        # no cache, MHA
    (4, 2, 16, 7, 9, 0),       # GQA 2:1 with cache
    (8, 2, 4, 13, 6, 3),       # GQA 4:1, observation window
    (2, 1, 32, 1, 1, 0),       # single-row chunk
    (6, 3, 8, 20, 17, 1),      # window of one row
])
def test_matches_materialised_softmax(Hq, Hkv, d, M, Ct, W):
    rng = np.random.default_rng(100 + Hq + M)
    q, k, v = rand_case(rng, Hq, Hkv, d, M, Ct)
    scale = 1.0 / math.sqrt(d)
    o, l, s = oracle.attend_score(q, k, v, M, scale, W=W)
    o2, l2, s2 = brute_force(q, k, v, M, scale, W)
    np.testing.assert_allclose(o, o2, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(l, l2, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(s[:, :M + Ct], s2[:, :M + Ct], rtol=1e-12, atol=1e-13)
    assert np.all(s[:, M + Ct:] == 0)


@pytest.mark.parametrize("M", [0, 11])
def test_matches_torch_sdpa(M):
    """M = 0 is plain causal attention; with a cache the mask is bottom-right aligned."""
    rng = np.random.default_rng(5)
    Hq, Hkv, d, Ct = 6, 2, 16, 10
    q, k, v = rand_case(rng, Hq, Hkv, d, M, Ct, extra_cap=0)
    scale = 0.37
    o, _, _ = oracle.attend_score(q, k, v, M, scale)
    tq = torch.from_numpy(q).double()[None]
    tk = torch.from_numpy(k).double().repeat_interleave(Hq // Hkv, dim=0)[None]
    tv = torch.from_numpy(v).double().repeat_interleave(Hq // Hkv, dim=0)[None]
    if M == 0:
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    else:
        n = M + Ct
        mask = torch.arange(n)[None, :] <= (M + torch.arange(Ct))[:, None]
        ref = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, attn_mask=mask, scale=scale)
    np.testing.assert_allclose(o, ref[0].numpy(), rtol=1e-10, atol=1e-12)


def load_uniform_golden():
    cases = []
    with open(os.path.join(GOLDEN, "uniform_attention_scores.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            head, vals = line.split(":")
            M, Ct, W, G = (int(x) for x in head.split())
            cases.append((M, Ct, W, G, [float(x) for x in vals.split()]))
    return cases


@pytest.mark.parametrize("case", load_uniform_golden(), ids=lambda c: f"M{c[0]}C{c[1]}W{c[2]}G{c[3]}")
def test_uniform_attention_closed_form(case):
    """Q = 0 makes every visible key equally likely: p_ij = 1/(M+i+1).

    Then out_i is the running mean of V and score_j = G * sum over observing rows that see j of
    1/(M+i+1).  The expected scores in the golden file were produced with exact rational
    arithmetic by tests/golden/make_uniform_golden.py (which calls nothing but `fractions`).
    """
    M, Ct, W, G, expect = case
    rng = np.random.default_rng(9)
    Hkv, d = 2, 4
    q, k, v = rand_case(rng, Hkv * G, Hkv, d, M, Ct)
    q[:] = 0
    o, l, s = oracle.attend_score(q, k, v, M, 0.5, W=W)
    n = M + Ct
    np.testing.assert_allclose(s[0, :n], np.array(expect), rtol=1e-13)
    np.testing.assert_allclose(s[1, :n], np.array(expect), rtol=1e-13)
    csum = np.cumsum(v[:, :n].astype(np.float64), axis=1)
    for i in range(Ct):
        mean = csum[:, M + i] / (M + i + 1)
        for h in range(Hkv * G):
            np.testing.assert_allclose(o[h, i], mean[h // G], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(l[:, i], math.log(M + i + 1), rtol=1e-13)


def test_total_mass_and_nonnegativity():
    rng = np.random.default_rng(1)
    Hq, Hkv, d, M, Ct, W = 8, 2, 8, 30, 25, 10
    q, k, v = rand_case(rng, Hq, Hkv, d, M, Ct)
    _, _, s = oracle.attend_score(q, k, v, M, 0.3, W=W)
    assert np.all(s >= 0)
    np.testing.assert_allclose(s.sum(axis=1), (Hq // Hkv) * W, rtol=1e-12)


def test_dominant_key_collects_every_row_that_sees_it():
    rng = np.random.default_rng(2)
    Hq, Hkv, d, M, Ct = 4, 2, 8, 6, 12
    q, k, v = rand_case(rng, Hq, Hkv, d, M, Ct)
    q[:] = np.abs(q) + 0.5
    jc, jn = 2, M + 4                      # one cache key, one chunk key
    k[:, :M + Ct] *= 0.01
    k[:, jc] = 100.0
    _, _, s = oracle.attend_score(q, k, v, M, 1.0)
    G = Hq // Hkv
    np.testing.assert_allclose(s[:, jc], G * Ct, rtol=1e-9)
    k[:, jc] = 0.0
    k[:, jn] = 100.0
    _, _, s = oracle.attend_score(q, k, v, M, 1.0)
    np.testing.assert_allclose(s[:, jn], G * (Ct - 4), rtol=1e-9)   # rows 4..Ct-1 see chunk key 4


def test_cache_permutation_and_duplicates():
    rng = np.random.default_rng(3)
    Hq, Hkv, d, M, Ct = 4, 2, 8, 16, 8
    q, k, v = rand_case(rng, Hq, Hkv, d, M, Ct, extra_cap=0)
    k[:, 9] = k[:, 3]                       # duplicate cache key: bit-equal scores
    o, l, s = oracle.attend_score(q, k, v, M, 0.4)
    assert np.array_equal(s[:, 9], s[:, 3])
    perm = rng.permutation(M)
    k2, v2 = k.copy(), v.copy()
    k2[:, :M] = k[:, perm]
    v2[:, :M] = v[:, perm]
    o2, l2, s2 = oracle.attend_score(q, k2, v2, M, 0.4)
    np.testing.assert_allclose(o2, o, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(l2, l, rtol=1e-12)
    np.testing.assert_allclose(s2[:, :M], s[:, perm], rtol=1e-11)
    np.testing.assert_allclose(s2[:, M:], s[:, M:], rtol=1e-11)


def test_accumulate_adds_to_previous_scores():
    rng = np.random.default_rng(4)
    q, k, v = rand_case(rng, 2, 1, 4, 5, 6)
    _, _, s = oracle.attend_score(q, k, v, 5, 0.5)
    prev = rng.random(s.shape)
    _, _, s2 = oracle.attend_score(q, k, v, 5, 0.5, accumulate=True, score_in=prev)
    np.testing.assert_allclose(s2[:, :11], prev[:, :11] + s[:, :11], rtol=1e-13)
    np.testing.assert_array_equal(s2[:, 11:], prev[:, 11:])


def test_sampled_rows_equal_full_pass():
    rng = np.random.default_rng(6)
    Hq, Hkv, d, M, Ct = 4, 2, 8, 9, 14
    q, k, v = rand_case(rng, Hq, Hkv, d, M, Ct)
    o, l, _ = oracle.attend_score(q, k, v, M, 0.2)
    rh = np.array([0, 3, 1, 2], np.int32)
    ri = np.array([0, 13, 7, 5], np.int32)
    o2, l2 = oracle.attend_rows(q, k, v, M, 0.2, rh, ri)
    np.testing.assert_array_equal(o2, o[rh, ri])
    np.testing.assert_array_equal(l2, l[rh, ri])


def test_sampled_row_score_is_the_mass_of_those_rows():
    """Zero queries give a closed-form share; the sampled rows add their own probabilities."""
    rng = np.random.default_rng(8)
    Hq, Hkv, d, M, Ct = 4, 2, 8, 7, 11
    q, k, v = rand_case(rng, Hq, Hkv, d, M, Ct)
    rh = np.array([0, 1, 3, 2, 0], np.int32)
    ri = np.array([0, 10, 4, 4, 6], np.int32)
    keep = np.zeros((Hq, Ct), bool)
    keep[rh, ri] = True
    q[~keep] = 0.0
    _, _, full = oracle.attend_score(q, k, v, M, 0.3)
    _, _, part = oracle.attend_rows(q, k, v, M, 0.3, rh, ri, want_score=True)
    uniform = np.zeros_like(full)
    for h in range(Hq):
        for i in range(Ct):
            if not keep[h, i]:
                uniform[h // 2, :M + i + 1] += 1.0 / (M + i + 1)
    np.testing.assert_allclose(part + uniform, full, rtol=1e-12, atol=1e-14)
    # sampling every row reproduces the full score
    hh, ii = np.meshgrid(np.arange(Hq), np.arange(Ct), indexing="ij")
    _, _, allrows = oracle.attend_rows(q, k, v, M, 0.3, hh.ravel(), ii.ravel(), want_score=True)
    np.testing.assert_allclose(allrows, full, rtol=1e-12, atol=1e-14)


def test_bad_arguments_rejected():
    rng = np.random.default_rng(7)
    q, k, v = rand_case(rng, 3, 2, 4, 2, 3)      # Hq % Hkv != 0
    with pytest.raises(ValueError):
        oracle.attend_score(q, k, v, 2, 1.0)
    q, k, v = rand_case(rng, 2, 2, 4, 2, 3)
    with pytest.raises(ValueError):
        oracle.attend_score(q, k, v, 50, 1.0)    # cap < M + Ct

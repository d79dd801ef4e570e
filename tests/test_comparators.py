"""CPU tests of the comparators themselves (tests/helpers.py): on the adversarial workload, whose
four sink keys carry scores thousands of times the median, a wrong score for an ORDINARY key must
fail, and the selection band must leave almost nothing undecided.  Mistakes are planted in copies
of the oracle's own numbers; no GPU is involved."""
import numpy as np
import pytest

import oracle
from helpers import (LAST_BAND, assert_close, assert_scores_close, assert_selection_within_band,
                     band_sets, robust_scale, to_np)
from paper_2506_01215_amd import synth


@pytest.fixture(scope="module")
def adversarial_scores():
    """Oracle scores of the scaled workload 5: chunk 0 (empty cache) and chunk 1 over a cache that
    holds the sinks (the first B rows of chunk 0)."""
    cfg = synth.scaled(synth.STREAMS[5], L=5 * 1024 + 17, C=1024, B=384)
    plan = synth.adversarial_plan(cfg)
    q0, k0, v0 = synth.chunk_qkv(cfg, 0, 0, plan=plan)
    q1, k1, v1 = synth.chunk_qkv(cfg, 0, 1, plan=plan)
    _, _, s0 = oracle.attend_score(to_np(q0), to_np(k0), to_np(v0), 0, cfg.scale)
    K = np.concatenate([to_np(k0)[:, :cfg.B], to_np(k1)], axis=1)
    V = np.concatenate([to_np(v0)[:, :cfg.B], to_np(v1)], axis=1)
    _, _, s1 = oracle.attend_score(to_np(q1), K, V, cfg.B, cfg.scale)
    return cfg, s0, s1


def test_sinks_dominate_the_plain_rms_but_not_the_robust_scale(adversarial_scores):
    cfg, s0, s1 = adversarial_scores
    for s in (s0, s1):
        for g in range(cfg.n_kv_heads):
            row = s[g]
            med = np.median(row)
            rms = np.sqrt(np.mean(row ** 2))
            assert row[:4].min() > 100 * med                      # the planted sinks
            assert rms > 20 * med                                  # whole-row RMS: useless as a floor
            assert robust_scale(row) < 3 * med                     # typical-candidate scale


@pytest.mark.parametrize("factor", [1.5, 0.5, 1.1])
def test_wrong_scores_of_ordinary_keys_fail(adversarial_scores, factor):
    cfg, s0, s1 = adversarial_scores
    for s in (s0, s1):
        assert_scores_close(s, s, 2e-2, "identity")
        bad = s.copy()
        bad[:, 4:] *= factor                                       # every non-sink score wrong
        with pytest.raises(AssertionError):
            assert_scores_close(bad, s, 2e-2, "planted")
        one = s.copy()
        one[3, 700] = 0.0                                          # one ordinary key loses its score
        assert s[3, 700] > 0.02
        with pytest.raises(AssertionError):
            assert_scores_close(one, s, 2e-2, "planted single")
    # the whole-tensor rule alone lets the same error on the typical keys through (its floor is
    # 3.4 x the median score here): that is why score comparisons use the robust floor
    bad = s0.copy()
    typical = s0 < 3 * np.median(s0, axis=1, keepdims=True)
    assert typical.mean() > 0.8
    bad[typical] *= factor
    assert_close(bad, s0, 2e-2, "whole-tensor rule")
    with pytest.raises(AssertionError):
        assert_scores_close(bad, s0, 2e-2, "planted, typical keys only")


def test_small_relative_noise_passes(adversarial_scores):
    _, s0, _ = adversarial_scores
    rng = np.random.default_rng(0)
    assert_scores_close(s0 * (1 + 5e-3 * rng.standard_normal(s0.shape)), s0, 2e-2, "noise")


def test_band_decides_almost_every_candidate(adversarial_scores):
    cfg, s0, s1 = adversarial_scores
    for s in (s0, s1):
        n = s.shape[1]
        for g in range(cfg.n_kv_heads):
            exact, must, never = band_sets(s[g], cfg.B, 2e-2)
            assert must.sum() + never.sum() > 0.9 * n
            assert must.sum() <= cfg.B <= n - never.sum()
            assert assert_selection_within_band(exact, s[g], cfg.B, 2e-2) == 0
            assert LAST_BAND["decided"] > 0.9 and LAST_BAND["tight_violations"] == 0


def test_band_rejects_a_swap_of_a_clear_winner_for_a_clear_loser(adversarial_scores):
    cfg, s0, _ = adversarial_scores
    s = s0[0]
    exact, must, never = band_sets(s, cfg.B, 2e-2)
    winner = int(np.flatnonzero(must)[-1])
    loser = int(np.flatnonzero(never)[0])
    swapped = np.sort(np.concatenate([exact[exact != winner], [loser]]))
    with pytest.raises(AssertionError):
        assert_selection_within_band(swapped, s, cfg.B, 2e-2)
    # the median candidate is a clear loser and the score just above the threshold a clear winner
    order = np.argsort(-s, kind="stable")
    assert never[order[len(s) // 2]] and must[order[cfg.B // 2]]


def test_band_accepts_only_exact_ties_when_threshold_is_zero():
    s = np.array([3.0, 0.0, 0.0, 2.0, 0.0, -1.0])
    assert assert_selection_within_band(np.array([0, 1, 3]), s, 3, 2e-2) == 0
    assert assert_selection_within_band(np.array([0, 3, 4]), s, 3, 2e-2) == 1    # another zero: in band
    with pytest.raises(AssertionError):
        assert_selection_within_band(np.array([0, 3, 5]), s, 3, 2e-2)


def test_threaded_oracle_front_end_equals_the_plain_call():
    """oracle_kv_heads_dense only spreads rows over threads: same numbers as oracle.attend_score."""
    from helpers import oracle_kv_heads_dense
    rng = np.random.default_rng(3)
    Hq, Hkv, d, M, Ct = 8, 4, 32, 37, 53
    q = rng.standard_normal((Hq, Ct, d)).astype(np.float32)
    K = rng.standard_normal((Hkv, M + Ct + 3, d)).astype(np.float32)
    V = rng.standard_normal((Hkv, M + Ct + 3, d)).astype(np.float32)
    o_ref, l_ref, s_ref = oracle.attend_score(q, K, V, M, 0.2)
    for heads in ([2], [0, 3]):
        o, l, s = oracle_kv_heads_dense(q, K, V, M, 0.2, heads, threads=3)
        qh = np.concatenate([np.arange(g * 2, g * 2 + 2) for g in heads])
        np.testing.assert_array_equal(o, o_ref[qh])
        np.testing.assert_array_equal(l, l_ref[qh])
        np.testing.assert_allclose(s, s_ref[heads][:, :M + Ct], rtol=1e-13, atol=0)

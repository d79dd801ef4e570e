"""GPU parity: reform_chunk_attend_score against the fp64 CPU oracle, element by element."""
import math

import numpy as np
import pytest
import torch

import oracle
from helpers import RTOL, assert_close, assert_scores_close, to_np
from paper_2506_01215_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make(Hq, Hkv, d, M, Ct, dtype, seed, extra_cap=5, kscale=1.0):
    g = torch.Generator().manual_seed(seed)
    cap = M + Ct + extra_cap
    q = torch.randn((Hq, Ct, d), generator=g).to(dtype)
    k = (torch.randn((Hkv, cap, d), generator=g) * kscale).to(dtype)
    v = torch.randn((Hkv, cap, d), generator=g).to(dtype)
    # rows past n must never influence a result
    k[:, M + Ct:] = float("nan")
    v[:, M + Ct:] = float("nan")
    return q, k, v


def run_case(q, k, v, M, scale, W=0, dtype=None):
    dtype = q.dtype
    print(f"[attend] dtype={dtype} q={tuple(q.shape)} kv={tuple(k.shape)} M={M} W={W}", flush=True)
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    out, lse, score = binding.reform_chunk_attend_score(qd, kd, vd, M, scale, obs_window=W)
    torch.cuda.synchronize()
    o_ref, l_ref, s_ref = oracle.attend_score(to_np(q), to_np(k), to_np(v), M, scale, W=W)
    n = M + q.shape[1]
    rtol = RTOL[dtype]
    assert_close(to_np(out), o_ref, rtol, "out")
    assert_close(to_np(lse), l_ref, rtol, "lse")
    assert_scores_close(to_np(score)[:, :n], s_ref[:, :n], rtol, "score")
    assert np.all(to_np(score)[:, n:] == 0), "score written past n"
    G = q.shape[0] // k.shape[0]
    Weff = q.shape[1] if W == 0 else W
    np.testing.assert_allclose(to_np(score)[:, :n].sum(axis=1), G * Weff, rtol=10 * rtol)
    return out, lse, score


@pytest.mark.parametrize("Hq,Hkv,d,M,Ct,W", [
    (4, 4, 64, 0, 128, 0),        # workload 1, first chunk
    (4, 4, 64, 256, 128, 0),      # workload 1, steady state
    (8, 2, 128, 77, 53, 0),       # GQA, ragged
    (6, 3, 32, 10, 70, 16),       # observation window, odd head_dim for fp32
    (2, 2, 64, 3, 1, 0),          # single-row chunk
])
def test_fp32_matches_oracle(Hq, Hkv, d, M, Ct, W):
    q, k, v = make(Hq, Hkv, d, M, Ct, torch.float32, 11 + M + Ct)
    run_case(q, k, v, M, 1.0 / math.sqrt(d), W)


@pytest.mark.parametrize("Hq,Hkv,d,M,Ct,W", [
    (8, 2, 128, 300, 200, 0),     # GQA 4:1, several key tiles, ragged rows and keys
    (4, 4, 64, 0, 130, 0),        # MHA, head_dim 64, no cache
    (4, 4, 128, 0, 64, 0),        # exactly one tile
    (16, 4, 128, 1000, 517, 128), # observation window smaller than the chunk
    (8, 8, 128, 4096, 17, 0),     # 17-row ragged tail over a full cache (workload 5's last chunk)
    (8, 4, 128, 130, 257, 0),     # GQA 2:1
    (16, 2, 64, 65, 63, 5),       # GQA 8:1
    (2, 2, 128, 1, 1, 0),         # smallest
])
def test_bf16_matches_oracle(Hq, Hkv, d, M, Ct, W):
    q, k, v = make(Hq, Hkv, d, M, Ct, torch.bfloat16, 23 + M + Ct)
    run_case(q, k, v, M, 1.0 / math.sqrt(d), W)


def test_bf16_key_norm_spread():
    """Keys with log-normal norms (workload 2): large logits, strongly peaked rows."""
    g = torch.Generator().manual_seed(5)
    Hq, Hkv, d, M, Ct = 8, 2, 128, 500, 260
    q, k, v = make(Hq, Hkv, d, M, Ct, torch.bfloat16, 6)
    z = torch.randn((1, k.shape[1], 1), generator=g)
    k = (k.float() * torch.exp(0.5 * z)).to(torch.bfloat16)
    k[:, M + Ct:] = float("nan")
    run_case(q, k, v, M, 1.0 / math.sqrt(d))


def test_strided_q_and_out():
    """q / out given as [Ct, Hq, d] storage viewed as [Hq, Ct, d] (what a QKV projection emits)."""
    Hq, Hkv, d, M, Ct = 8, 2, 128, 100, 90
    q, k, v = make(Hq, Hkv, d, M, Ct, torch.bfloat16, 31)
    qs = q.permute(1, 0, 2).contiguous().to(DEV).permute(1, 0, 2)
    assert not qs.is_contiguous()
    out = torch.empty((Ct, Hq, d), dtype=torch.bfloat16, device=DEV).permute(1, 0, 2)
    scale = 1.0 / math.sqrt(d)
    o, lse, score = binding.reform_chunk_attend_score(qs, k.to(DEV), v.to(DEV), M, scale, out=out)
    torch.cuda.synchronize()
    o_ref, l_ref, s_ref = oracle.attend_score(to_np(q), to_np(k), to_np(v), M, scale)
    assert_close(to_np(o), o_ref, 2e-2, "out")
    assert_scores_close(to_np(score)[:, :M + Ct], s_ref[:, :M + Ct], 2e-2, "score")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_accumulate_and_attention_only(dtype):
    Hq, Hkv, d, M, Ct = 4, 2, 64, 40, 50
    q, k, v = make(Hq, Hkv, d, M, Ct, dtype, 41)
    scale = 0.125
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    prev = torch.rand((Hkv, k.shape[1]), device=DEV)
    score = prev.clone()
    binding.reform_chunk_attend_score(qd, kd, vd, M, scale, accumulate=True, score=score)
    out2, lse2, none = binding.reform_chunk_attend_score(qd, kd, vd, M, scale, want_score=False)
    torch.cuda.synchronize()
    assert none is None
    o_ref, l_ref, s_ref = oracle.attend_score(to_np(q), to_np(k), to_np(v), M, scale, accumulate=True,
                                              score_in=to_np(prev))
    n = M + Ct
    assert_scores_close(to_np(score)[:, :n], s_ref[:, :n], RTOL[dtype], "score+=")
    assert torch.equal(score[:, n:], prev[:, n:])
    assert_close(to_np(out2), o_ref, RTOL[dtype], "out (attention only)")


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_duplicate_cache_keys_tie_exactly_and_runs_are_bitwise_reproducible(dtype):
    Hq, Hkv, d, M, Ct = 8, 2, 128, 700, 300
    q, k, v = make(Hq, Hkv, d, M, Ct, dtype, 51)
    # duplicates far apart: different tiles, waves and lanes
    pairs = [(3, 640), (64, 65), (100, 333), (255, 256), (0, 699)]
    for a, b in pairs:
        k[:, b] = k[:, a]
    qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
    o1, l1, s1 = binding.reform_chunk_attend_score(qd, kd, vd, M, 0.09)
    o2, l2, s2 = binding.reform_chunk_attend_score(qd, kd, vd, M, 0.09)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(l1, l2) and torch.equal(s1, s2)
    for a, b in pairs:
        assert torch.equal(s1[:, a], s1[:, b]), f"duplicate keys {a},{b} scored differently"


def test_uniform_attention_closed_form_large():
    """Q = 0: p = 1/(M+i+1); out is the running mean of V, score a harmonic sum.  Checked at a
    size spanning many tiles with ragged ends, against numpy cumulative sums in fp64."""
    Hq, Hkv, d, M, Ct, W = 8, 2, 128, 5000, 3001, 1234
    q, k, v = make(Hq, Hkv, d, M, Ct, torch.bfloat16, 61)
    q.zero_()
    out, lse, score = binding.reform_chunk_attend_score(q.to(DEV), k.to(DEV), v.to(DEV), M, 0.1,
                                                        obs_window=W)
    torch.cuda.synchronize()
    n = M + Ct
    i = np.arange(Ct)
    w = 1.0 / (M + i + 1.0)
    w_obs = np.where(i >= Ct - W, w, 0.0)
    tail = np.cumsum(w_obs[::-1])[::-1]                  # sum_{i' >= i} w_obs
    expect = np.concatenate([np.full(M, tail[0]), tail]) * (Hq // Hkv)
    assert_scores_close(to_np(score)[0, :n], expect, 2e-2, "score closed form")
    assert_scores_close(to_np(score)[1, :n], expect, 2e-2, "score closed form")
    vm = np.cumsum(to_np(v)[:, :n].astype(np.float64), axis=1)[:, M:] / (M + i + 1.0)[None, :, None]
    assert_close(to_np(out), np.repeat(vm, Hq // Hkv, axis=0), 2e-2, "running mean")
    assert_close(to_np(lse), np.broadcast_to(np.log(M + i + 1.0), (Hq, Ct)), 2e-2, "lse")

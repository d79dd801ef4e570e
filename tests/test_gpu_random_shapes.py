"""Seeded sweep over random small shapes for the three main calls, each case against the fp64
oracle: odd group sizes, chunk lengths and cache lengths around the tile sizes (32, 64, 256,
512), windows of every size, budgets from 1 to n-1, forced slots, several query counts."""
import math

import numpy as np
import pytest
import torch

import oracle
from helpers import RTOL, assert_close, assert_scores_close, assert_selection_within_band, numpy_union, to_np
from paper_2506_01215_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def pick_len(rng):
    """Lengths that cluster around tile boundaries."""
    base = int(rng.choice([1, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 255, 256, 257, 511, 513, 700]))
    return max(1, base + int(rng.integers(-1, 2)))


@pytest.mark.parametrize("seed", range(24))
def test_attend_score_random_shape(seed):
    rng = np.random.default_rng(1000 + seed)
    bf16 = seed % 3 != 0
    dtype = torch.bfloat16 if bf16 else torch.float32
    d = int(rng.choice([64, 128])) if bf16 else int(rng.choice([8, 32, 64, 100]))
    Hkv = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 3, 4, 5, 8]))
    Hq = Hkv * G
    Ct = pick_len(rng)
    M = 0 if rng.random() < 0.2 else pick_len(rng)
    W = 0 if rng.random() < 0.4 else int(rng.integers(1, Ct + 1))
    cap = M + Ct + int(rng.integers(0, 9))
    g = torch.Generator().manual_seed(seed)
    q = torch.randn((Hq, Ct, d), generator=g).to(dtype)
    k = (torch.randn((Hkv, cap, d), generator=g) * float(rng.choice([0.5, 1.0, 2.0]))).to(dtype)
    v = torch.randn((Hkv, cap, d), generator=g).to(dtype)
    scale = 1.0 / math.sqrt(d)
    print(f"[sweep attend] seed={seed} {dtype} Hq={Hq} Hkv={Hkv} d={d} M={M} Ct={Ct} W={W} cap={cap}", flush=True)
    out, lse, score = binding.reform_chunk_attend_score(q.to(DEV), k.to(DEV), v.to(DEV), M, scale, obs_window=W)
    torch.cuda.synchronize()
    o_ref, l_ref, s_ref = oracle.attend_score(to_np(q), to_np(k), to_np(v), M, scale, W=W)
    n = M + Ct
    assert_close(to_np(out), o_ref, RTOL[dtype], "out")
    assert_close(to_np(lse), l_ref, RTOL[dtype], "lse")
    assert_scores_close(to_np(score)[:, :n], s_ref[:, :n], RTOL[dtype], "score")


@pytest.mark.parametrize("seed", range(24))
def test_evict_random_shape(seed):
    rng = np.random.default_rng(2000 + seed)
    dtype = torch.bfloat16 if seed % 2 else torch.float32
    d = int(rng.choice([8, 16, 64, 96, 128, 256])) if dtype == torch.bfloat16 else int(rng.choice([4, 12, 64, 128]))
    Hkv = int(rng.integers(1, 6))
    n = int(rng.integers(2, 3000))
    B = int(rng.integers(1, n)) if rng.random() < 0.85 else n + int(rng.integers(0, 5))
    n_sink = int(rng.integers(0, min(B, 6) + 1)) if rng.random() < 0.5 else 0
    n_recent = int(rng.integers(0, B - n_sink + 1)) if rng.random() < 0.5 else 0
    cap = n + int(rng.integers(0, 20))
    g = torch.Generator().manual_seed(seed)
    k = torch.randn((Hkv, cap, d), generator=g).to(dtype)
    v = torch.randn((Hkv, cap, d), generator=g).to(dtype)
    if rng.random() < 0.5:
        score = torch.randint(0, 9, (Hkv, cap), generator=g).float() * 0.125       # heavy ties
    else:
        score = torch.randn((Hkv, cap), generator=g)                               # signed
    pos = torch.arange(cap, dtype=torch.int32).repeat(Hkv, 1).contiguous() + 11
    print(f"[sweep evict] seed={seed} {dtype} Hkv={Hkv} d={d} n={n} B={B} sink={n_sink} recent={n_recent}", flush=True)
    kd, vd, sd, pd = k.to(DEV), v.to(DEV), score.to(DEV), pos.to(DEV)
    kept = torch.full((Hkv, B), -1, dtype=torch.int32, device=DEV)
    new_len = binding.reform_evict_topk_compact(kd, vd, sd, n, B, n_sink, n_recent, pos=pd, kept_idx=kept)
    torch.cuda.synchronize()
    k2, v2, s2, p2, kept_ref = oracle.evict_compact(to_np(k), to_np(v), score.numpy().astype(np.float64),
                                                    pos.numpy(), n, B, n_sink, n_recent)
    assert new_len == min(n, B)
    np.testing.assert_array_equal(kept.cpu().numpy()[:, :new_len], kept_ref)
    np.testing.assert_array_equal(to_np(kd)[:, :new_len], k2[:, :new_len])
    np.testing.assert_array_equal(to_np(vd)[:, :new_len], v2[:, :new_len])
    np.testing.assert_array_equal(sd.cpu().numpy()[:, :new_len].astype(np.float64), s2[:, :new_len])
    np.testing.assert_array_equal(pd.cpu().numpy()[:, :new_len], p2[:, :new_len])
    np.testing.assert_array_equal(to_np(kd)[:, n:], to_np(k)[:, n:])


@pytest.mark.parametrize("seed", range(16))
def test_gather_random_shape(seed):
    rng = np.random.default_rng(3000 + seed)
    dtype = torch.bfloat16 if seed % 2 else torch.float32
    D = int(rng.choice([32, 64, 256, 1024])) if dtype == torch.bfloat16 else int(rng.choice([8, 24, 64, 256]))
    N = int(rng.integers(1, 9000))
    nq = int(rng.choice([1, 2, 3, 16, 17, 33]))
    k = int(rng.integers(1, N + 1))
    radius = int(rng.choice([0, 0, 1, 8, 64]))
    n_head = int(rng.integers(0, 4)) if rng.random() < 0.5 else 0
    n_tail = int(rng.integers(0, 4)) if rng.random() < 0.5 else 0
    g = torch.Generator().manual_seed(seed)
    emb = torch.randn((N, D), generator=g).to(dtype)
    qry = torch.randn((nq, D), generator=g).to(dtype)
    print(f"[sweep gather] seed={seed} {dtype} N={N} D={D} nq={nq} k={k} r={radius} keep={n_head}/{n_tail}", flush=True)
    idx, sc, uni, cnt = binding.reform_gather_topk(emb.to(DEV), qry.to(DEV), k, radius, n_head, n_tail)
    torch.cuda.synchronize()
    sim_ref = oracle.cosine(to_np(emb), to_np(qry))
    idx_h = idx.cpu().numpy()
    for qi in range(nq):
        assert_selection_within_band(idx_h[qi], sim_ref[qi], k, RTOL[dtype], f"top-k q={qi}")
        assert_close(sc.cpu().numpy()[qi], sim_ref[qi][idx_h[qi]], RTOL[dtype], f"scores q={qi}")
    got = uni.cpu().numpy()[:int(cnt.item())]
    np.testing.assert_array_equal(got, numpy_union(idx_h, N, radius, n_head, n_tail))


@pytest.mark.parametrize("seed", range(16))
def test_selection_random_sizes_across_paths(seed):
    """Evict (odd seeds) and gather (even seeds) at random sizes from 2 to 200000 candidates per
    row, so that every variant of the selection is hit (one launch with 4 to 32 keys per lane,
    several launches), with exact ties, forced slots and unaligned row pitches.  The integer
    results must match exactly (the gather on the GPU's own similarity values)."""
    rng = np.random.default_rng(7000 + seed)
    g = torch.Generator().manual_seed(seed)
    if seed % 2:
        Hkv = int(rng.integers(1, 4))
        n = int([rng.integers(2, 5000), rng.integers(4000, 9000), rng.integers(16000, 17000),
                 rng.integers(30000, 34000), rng.integers(60000, 70000), rng.integers(100000, 140000)][(seed // 2) % 6])
        B = int(rng.integers(1, n))
        d = int(rng.choice([8, 64]))
        cap = n + int(rng.integers(0, 9))
        ns = int(rng.integers(0, min(B, 300) + 1)) if rng.random() < 0.4 else 0
        nr = int(rng.integers(0, min(B - ns, 300) + 1)) if rng.random() < 0.4 else 0
        k = torch.randn((Hkv, cap, d), generator=g).bfloat16()
        v = torch.randn((Hkv, cap, d), generator=g).bfloat16()
        if rng.random() < 0.5:
            score = torch.randint(0, int(rng.choice([2, 7, 1000])), (Hkv, cap), generator=g).float() * 0.25 - 1.0
        else:
            score = torch.randn((Hkv, cap), generator=g)
        pos = torch.arange(cap, dtype=torch.int32).repeat(Hkv, 1).contiguous()
        kd, vd, sd, pd = k.to(DEV), v.to(DEV), score.to(DEV), pos.to(DEV)
        kept = torch.full((Hkv, B), -1, dtype=torch.int32, device=DEV)
        print(f"[sweep select/evict] seed={seed} Hkv={Hkv} n={n} B={B} d={d} cap={cap} sink={ns} recent={nr}", flush=True)
        binding.reform_evict_topk_compact(kd, vd, sd, n, B, ns, nr, pos=pd, kept_idx=kept)
        torch.cuda.synchronize()
        k2, v2, s2, p2, kept_ref = oracle.evict_compact(to_np(k), to_np(v), to_np(score).astype(np.float64),
                                                        pos.numpy(), n, B, ns, nr)
        np.testing.assert_array_equal(kept.cpu().numpy(), kept_ref)
        np.testing.assert_array_equal(to_np(kd)[:, :B], k2[:, :B])
        np.testing.assert_array_equal(to_np(vd)[:, :B], v2[:, :B])
        np.testing.assert_array_equal(sd.cpu().numpy()[:, :B].astype(np.float64), s2[:, :B])
        np.testing.assert_array_equal(pd.cpu().numpy()[:, :B], p2[:, :B])
    else:
        N = int([rng.integers(1, 5000), rng.integers(8000, 9000), rng.integers(30000, 36000),
                 rng.integers(60000, 200000)][(seed // 2) % 4])
        D = int(rng.choice([32, 64]))
        nq = int(rng.integers(1, 20))
        kk = int(rng.integers(1, N + 1)) if rng.random() < 0.3 else int(rng.integers(1, max(2, N // 10)))
        r = int(rng.choice([0, 1, 8]))
        emb = torch.randn((N, D), generator=g).bfloat16()
        if rng.random() < 0.5:                                    # duplicated rows: exact ties
            emb[torch.from_numpy(rng.integers(0, N, size=max(1, N // 3)))] = emb[0].clone()
        qry = torch.randn((nq, D), generator=g).bfloat16()
        n_tail = 2 if N > 2 else 0
        print(f"[sweep select/gather] seed={seed} N={N} D={D} nq={nq} k={kk} r={r}", flush=True)
        ti, ts, ui, uc = binding.reform_gather_topk(emb.to(DEV), qry.to(DEV), kk, r, 1, n_tail)
        sim = binding.reform_gather_similarity(emb.to(DEV), qry.to(DEV))
        torch.cuda.synchronize()
        simn = sim.cpu().numpy()
        for q in range(nq):
            ref = np.sort(np.lexsort((np.arange(N), -simn[q].astype(np.float64)))[:kk])
            np.testing.assert_array_equal(ti[q].cpu().numpy(), ref)
            np.testing.assert_array_equal(ts[q].cpu().numpy(), simn[q][ref])
        un = numpy_union(ti.cpu().numpy(), N, r, 1, n_tail)
        assert int(uc.item()) == len(un)
        np.testing.assert_array_equal(ui[:len(un)].cpu().numpy(), un)

"""GPU parity at full size with DENSE queries, element by element against the fp64 oracle.

  * workload 3: one steady layer-step (M = C = 32768, 32/8 heads, the shape bench.py times,
    every chunk row observing): out, lse and the whole 65536-entry score row of one KV group,
    then the selection -- exact on the GPU's own scores for every head, banded on the oracle's;
  * workload 2: the whole recurrence, all 16 chunks at C = B = 8192, the oracle following two KV
    heads in lock-step;
  * workload 5: the whole recurrence, all 65 chunks (the last one 17 rows), the oracle checking
    chunks 0, 1, 2, 31, 63 and the tail on all 8 heads.

Inputs are generated on the device by the seeded generators and every token's original K/V row
is kept in a device-side store; the oracle receives copies of those inputs.  Lock-step: before a
checked chunk the oracle's cache is rebuilt from the store rows of the token ids the GPU holds,
so only the identity of retained tokens ever comes from the GPU, never a floating-point value.
The oracle's rows are spread over host threads (helpers.oracle_kv_heads_dense)."""
import time

import numpy as np
import pytest
import torch

from helpers import (RTOL, BandTally, assert_close, assert_scores_close, assert_selection_within_band,
                     oracle_kv_heads_dense, to_np)
from paper_2506_01215_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def exact_on_own_scores(kept_row, score_row, n, B, n_sink=0, n_recent=0):
    s = score_row[:n].astype(np.float64)
    forced = np.zeros(n, bool)
    forced[:n_sink] = True
    if n_recent:
        forced[n - n_recent:] = True
    key = np.where(forced, np.inf, s)
    want = np.sort(np.lexsort((np.arange(n), -key))[:B])
    np.testing.assert_array_equal(kept_row, want)


def check_against_oracle(tag, q, Kpre, Vpre, M, scale, kv_heads, G, out, lse, score_gpu, kept_h, n, B, rtol, tally):
    """q [Hq,Ct,d] device; Kpre, Vpre [len(kv_heads), n, d] device: the pre-step cache of those heads."""
    t0 = time.time()
    Hkv_all = score_gpu.shape[0]
    qn = to_np(q)
    Kn = np.zeros((Hkv_all, n, qn.shape[2]), np.float32)
    Vn = np.zeros_like(Kn)
    Kn[kv_heads] = to_np(Kpre)
    Vn[kv_heads] = to_np(Vpre)
    o_ref, l_ref, s_ref = oracle_kv_heads_dense(qn, Kn, Vn, M, scale, kv_heads)
    qh = np.concatenate([np.arange(g * G, (g + 1) * G) for g in kv_heads])
    assert_close(to_np(out[qh]), o_ref, rtol, f"{tag}: out", row_floor=True)
    assert_close(to_np(lse[qh]), l_ref, rtol, f"{tag}: lse")
    assert_scores_close(score_gpu[kv_heads][:, :n], s_ref, rtol, f"{tag}: score")
    rel = np.abs(score_gpu[kv_heads][:, :n] - s_ref) / np.maximum(np.abs(s_ref), 1e-30)
    big = s_ref > np.median(s_ref, axis=1, keepdims=True)
    new_len = min(n, B)
    if n > B:
        for a, g in enumerate(kv_heads):
            assert_selection_within_band(kept_h[g, :new_len], s_ref[a], new_len, rtol, f"{tag}: kept head {g}")
            tally.add()
    print(f"[dense] {tag}: KV heads {list(kv_heads)} checked in {time.time() - t0:.1f} s; max relative score "
          f"error over the upper half {rel[big].max():.2e}", flush=True)


def test_workload3_steady_step_dense_one_kv_group():
    cfg = synth.STREAMS[3]
    Hq, Hkv, d, B = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.B
    G = Hq // Hkv
    layer, g0 = 2, 5
    _, k0, v0 = synth.chunk_qkv(cfg, layer, 0, device=DEV)
    q, k1, v1 = synth.chunk_qkv(cfg, layer, 1, device=DEV)
    M, Ct = B, q.shape[1]
    n = M + Ct
    Kd = torch.cat([k0[:, :M], k1], dim=1).contiguous()
    Vd = torch.cat([v0[:, :M], v1], dim=1).contiguous()
    Kpre, Vpre = Kd[[g0]].clone(), Vd[[g0]].clone()
    print(f"[dense] {cfg.name}: M={M} Ct={Ct} W=C, oracle on KV head {g0}", flush=True)
    out, lse, score = binding.reform_chunk_attend_score(q, Kd, Vd, M, cfg.scale)
    score_gpu = score.cpu().numpy()
    kept = torch.full((Hkv, B), -1, dtype=torch.int32, device=DEV)
    new_len = binding.reform_evict_topk_compact(Kd, Vd, score, n, B, kept_idx=kept)
    torch.cuda.synchronize()
    kept_h = kept.cpu().numpy()
    for g in range(Hkv):
        exact_on_own_scores(kept_h[g], score_gpu[g], n, B)
    np.testing.assert_allclose(score_gpu[:, :n].sum(axis=1), G * Ct, rtol=1e-4)
    assert torch.equal(Kd[g0, :new_len], Kpre[0][kept[g0].long()])
    tally = BandTally()
    check_against_oracle("workload 3 steady step", q, Kpre, Vpre, M, cfg.scale, [g0], G, out, lse, score_gpu,
                         kept_h, n, B, RTOL[cfg.dtype], tally)
    print(f"[dense] workload 3 steady step: {tally}", flush=True)


def lockstep_full(cfg, oracle_heads, check_chunks):
    Hq, Hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    G = Hq // Hkv
    cap, B = cfg.capacity, cfg.B
    rtol = RTOL[cfg.dtype]
    plan = synth.adversarial_plan(cfg) if cfg.kind == "adversarial" else None
    Kd = torch.zeros((Hkv, cap, d), dtype=cfg.dtype, device=DEV)
    Vd = torch.zeros_like(Kd)
    pos = torch.full((Hkv, cap), -1, dtype=torch.int32, device=DEV)
    K_all = torch.zeros((Hkv, cfg.L, d), dtype=cfg.dtype, device=DEV)     # every token's original rows
    V_all = torch.zeros_like(K_all)
    oh = torch.tensor(list(oracle_heads), device=DEV)
    tally = BandTally()
    M = 0
    t_start = time.time()
    for t in range(cfg.n_chunks):
        q, k, v = synth.chunk_qkv(cfg, 0, t, device=DEV, plan=plan)
        Ct = q.shape[1]
        base = t * cfg.C
        n = M + Ct
        K_all[:, base:base + Ct] = k
        V_all[:, base:base + Ct] = v
        Kd[:, M:n] = k
        Vd[:, M:n] = v
        pos[:, M:n] = torch.arange(base, base + Ct, dtype=torch.int32, device=DEV)
        pos_before = pos[:, :n].long()
        checked = t in check_chunks
        if checked or t % 8 == 0:
            print(f"[dense] {cfg.name} chunk {t}/{cfg.n_chunks} M={M} Ct={Ct} "
                  f"({time.time() - t_start:.0f} s){' -- oracle' if checked else ''}", flush=True)
        if checked:
            idx = pos_before[oh].unsqueeze(-1).expand(-1, -1, d)
            Kpre = torch.gather(K_all[oh], 1, idx)                  # from the store, by token id
            Vpre = torch.gather(V_all[oh], 1, idx)
            assert torch.equal(Kpre, Kd[oh, :n]) and torch.equal(Vpre, Vd[oh, :n])
        out, lse, score = binding.reform_chunk_attend_score(q, Kd, Vd, M, cfg.scale)
        score_gpu = score.cpu().numpy()
        kept = torch.full((Hkv, B), -1, dtype=torch.int32, device=DEV)
        new_len = binding.reform_evict_topk_compact(Kd, Vd, score, n, B, pos=pos, kept_idx=kept)
        torch.cuda.synchronize()
        kept_h = kept.cpu().numpy()
        # every chunk: the selection is exact on the GPU's own scores and the right original rows moved
        kl = kept[:, :new_len].long()
        assert torch.equal(pos[:, :new_len].long(), torch.gather(pos_before, 1, kl))
        rows = pos[:, :new_len].long().unsqueeze(-1).expand(-1, -1, d)
        assert torch.equal(Kd[:, :new_len], torch.gather(K_all, 1, rows))
        assert torch.equal(Vd[:, :new_len], torch.gather(V_all, 1, rows))
        for g in range(Hkv):
            if n > B:
                exact_on_own_scores(kept_h[g, :new_len], score_gpu[g], n, B)
            else:
                np.testing.assert_array_equal(kept_h[g, :new_len], np.arange(n))
        np.testing.assert_allclose(score_gpu[:, :n].sum(axis=1), G * Ct, rtol=1e-4)
        if checked:
            check_against_oracle(f"{cfg.name} chunk {t}", q, Kpre, Vpre, M, cfg.scale, list(oracle_heads), G,
                                 out, lse, score_gpu, kept_h, n, B, rtol, tally)
        M = new_len
    print(f"[dense] {cfg.name}: {tally}", flush=True)
    return pos[:, :M].cpu().numpy(), plan


def test_workload2_full_recurrence_two_kv_heads_in_lockstep():
    cfg = synth.STREAMS[2]
    final, _ = lockstep_full(cfg, oracle_heads=(1, 6), check_chunks=set(range(cfg.n_chunks)))
    assert final.shape == (cfg.n_kv_heads, cfg.B)
    assert (np.diff(final, axis=1) > 0).all()                        # retained tokens stay in order


def test_workload5_full_recurrence_sampled_chunks_all_heads():
    cfg = synth.STREAMS[5]
    last = cfg.n_chunks - 1
    assert cfg.n_chunks == 65 and cfg.chunk_len(last) == 17
    final, plan = lockstep_full(cfg, oracle_heads=range(cfg.n_kv_heads), check_chunks={0, 1, 2, 31, 63, last})
    assert final.shape == (cfg.n_kv_heads, cfg.B)
    for g in range(cfg.n_kv_heads):
        assert set(range(4)) <= set(final[g].tolist()), "attention sinks were evicted"
    needles = set(plan["needle_pos"].tolist())
    survived = np.mean([len(needles & set(final[g].tolist())) for g in range(cfg.n_kv_heads)])
    print(f"[dense] workload 5: {survived:.1f} of 64 needles in the final cache, sinks kept on every head", flush=True)

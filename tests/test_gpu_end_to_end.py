"""The whole procedure of Alg. 1 on a small synthetic stream, every step through the C ABI:

    for each chunk (the last one is the query):            recurrent chunked forwarding
        for each layer:  attention + eviction score         reform_chunk_attend_score
                         save the selected head states      reform_embed_save_selected
                         compress the cache                 reform_evict_topk_compact
                         consecutive position ids           reform_rerotate_keys
    identify the significant inputs                         reform_gather_pooled
    gather them for recomputation                           reform_gather_rows

The oracle runs the same recurrence on its own data: its cache is compacted with the token choice
the GPU made (checked against the oracle's scores first), re-rotated by the oracle in fp64 and
stored as bf16 like the real cache; no floating-point value ever crosses from the GPU side.
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import RTOL, assert_close, assert_scores_close, assert_selection_within_band, to_np
from paper_2506_01215_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def as_bf16(x):
    """What a bf16 cache keeps of an fp64 result (round to nearest even, torch CPU conversion)."""
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).bfloat16().float().numpy()


def test_alg1_small_stream():
    n_layers, theta = 2, 10000.0
    base = synth.scaled(synth.STREAMS[2], L=5 * 512 + 64, C=512, B=512)     # 5 context chunks + a 64-token query
    Hq, Hkv, d, cap, B, C = base.n_q_heads, base.n_kv_heads, base.head_dim, base.capacity, base.B, base.C
    L, L_ctx = base.L, 5 * 512
    W, n_sink, n_recent = 128, 64, 64
    picks = [(0, "q", 5), (0, "k", 1), (1, "k", 6), (1, "v", 2)]            # (layer, state, head)
    D = d * len(picks)
    rtol = RTOL[torch.bfloat16]

    Kd = [torch.zeros((Hkv, cap, d), dtype=torch.bfloat16, device=DEV) for _ in range(n_layers)]
    Vd = [torch.zeros_like(Kd[0]) for _ in range(n_layers)]
    Ko = [np.zeros((Hkv, cap, d), np.float32) for _ in range(n_layers)]     # the oracle's own caches
    Vo = [np.zeros((Hkv, cap, d), np.float32) for _ in range(n_layers)]
    emb = torch.zeros((L, D), dtype=torch.bfloat16, device=DEV)
    emb_ref = np.zeros((L, D))
    kept = torch.empty((Hkv, B), dtype=torch.int32, device=DEV)
    M = 0
    for t in range(base.n_chunks):
        Ct = base.chunk_len(t)
        n = M + Ct
        Wt = min(W, Ct)
        for l in range(n_layers):
            q, k, v = synth.chunk_qkv(base, l, t)
            print(f"[alg1] chunk {t} layer {l} M={M} Ct={Ct}", flush=True)
            qd, kd, vd = q.to(DEV), k.to(DEV), v.to(DEV)
            Kd[l][:, M:n] = kd
            Vd[l][:, M:n] = vd
            Ko[l][:, M:n] = to_np(k)
            Vo[l][:, M:n] = to_np(v)
            out, lse, score = binding.reform_chunk_attend_score(qd, Kd[l], Vd[l], M, base.scale, obs_window=Wt)
            score_h = to_np(score)                      # the eviction compacts the score row in place
            states = {"q": qd, "k": kd, "v": vd}
            for seg, (pl, kind, head) in enumerate(picks):
                if pl == l:
                    binding.reform_embed_save_selected(states[kind][head], emb, t * C, seg * d)
                    oracle.embed_segment(to_np({"q": q, "k": k, "v": v}[kind][head]),
                                         emb_ref[t * C:t * C + Ct], seg * d)
            new_len = binding.reform_evict_topk_compact(Kd[l], Vd[l], score, n, B, n_sink, n_recent, kept_idx=kept)
            binding.reform_rerotate_keys(Kd[l], kept, new_len, theta)
            torch.cuda.synchronize()
            # ---- oracle: same chunk on its own cache
            o_ref, l_ref, s_ref = oracle.attend_score(to_np(q), Ko[l], Vo[l], M, base.scale, W=Wt)
            assert_close(to_np(out), o_ref, rtol, f"out chunk {t} layer {l}")
            assert_close(to_np(lse), l_ref, rtol, f"lse chunk {t} layer {l}")
            assert_scores_close(score_h[:, :n], s_ref[:, :n], rtol, f"score chunk {t} layer {l}")
            kept_h = kept.cpu().numpy()
            for g in range(Hkv):
                forced = list(range(min(n_sink, n))) + list(range(max(n - n_recent, 0), n)) if n > B else []
                assert_selection_within_band(kept_h[g, :new_len], s_ref[g, :n], new_len, rtol,
                                             f"kept chunk {t} layer {l} head {g}", forced)
                kg = kept_h[g, :new_len]
                Ko[l][g, :new_len] = as_bf16(oracle.rerotate_keys(Ko[l][g, kg], kg, theta))
                Vo[l][g, :new_len] = Vo[l][g, kg]
            assert_close(to_np(Kd[l])[:, :new_len], Ko[l][:, :new_len], rtol, f"cache keys after chunk {t} layer {l}")
            np.testing.assert_array_equal(to_np(Vd[l])[:, :new_len], Vo[l][:, :new_len])
        M = min(n, B)

    assert_close(to_np(emb), emb_ref, rtol, "embedding store")
    budget = 700
    ctx, qry = emb[:L_ctx].contiguous(), emb[L_ctx:].contiguous()
    sel, pooled = binding.reform_gather_pooled(ctx, qry, budget, 129, n_sink, n_recent)
    g = torch.Generator().manual_seed(3)
    table = torch.randn((L_ctx, 256), generator=g).bfloat16()
    rows = binding.reform_gather_rows(table.to(DEV), sel)
    torch.cuda.synchronize()
    _, p_ref, _ = oracle.gather_pooled(emb_ref[:L_ctx].astype(np.float32), emb_ref[L_ctx:].astype(np.float32),
                                       budget, 129, n_sink, n_recent)
    assert_close(pooled.cpu().numpy(), p_ref, rtol, "pooled significance scores")
    sel_h = sel.cpu().numpy()
    forced = list(range(n_sink)) + list(range(L_ctx - n_recent, L_ctx))
    assert_selection_within_band(sel_h, p_ref, budget, rtol, "significant inputs", forced)
    raw = lambda x: x.cpu().contiguous().view(torch.uint8).numpy().reshape(x.shape[0], -1)
    np.testing.assert_array_equal(raw(rows), oracle.gather_rows(raw(table), sel_h))

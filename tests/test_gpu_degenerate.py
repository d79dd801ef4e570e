"""Degenerate inputs of every call: nothing to do, everything selected, smallest shapes.  Each
must return REFORM_OK, leave untouched what it has no business touching, and agree with the
oracle where there is anything to compute."""
import numpy as np
import pytest
import torch

import oracle
from helpers import RTOL, assert_close, to_np
from paper_2506_01215_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_evict_with_no_candidates_and_with_exactly_the_budget():
    g = torch.Generator().manual_seed(0)
    k = torch.randn((2, 40, 64), generator=g).bfloat16().to(DEV)
    v = torch.randn((2, 40, 64), generator=g).bfloat16().to(DEV)
    score = torch.rand((2, 40), generator=g).to(DEV)
    k0, v0, s0 = k.clone(), v.clone(), score.clone()
    kept = torch.full((2, 16), -7, dtype=torch.int32, device=DEV)
    assert binding.reform_evict_topk_compact(k, v, score, 0, 16, kept_idx=kept) == 0     # empty cache
    torch.cuda.synchronize()
    assert torch.equal(k, k0) and torch.equal(v, v0) and torch.equal(score, s0)
    assert binding.reform_evict_topk_compact(k, v, score, 16, 16, kept_idx=kept) == 16   # n == B: keep all
    torch.cuda.synchronize()
    assert torch.equal(k, k0) and torch.equal(v, v0)
    assert (kept.cpu().numpy() == np.arange(16)[None, :]).all()
    assert binding.reform_evict_topk_compact(k, v, score, 17, 16, kept_idx=kept) == 16   # evict exactly one
    torch.cuda.synchronize()
    for h in range(2):
        want = oracle.evict_select(s0[h].cpu().numpy().astype(np.float64), 17, 16)
        np.testing.assert_array_equal(kept[h].cpu().numpy(), want)
        np.testing.assert_array_equal(to_np(k)[h, :16], to_np(k0)[h, want])


def test_gather_selecting_every_row_and_a_single_row():
    g = torch.Generator().manual_seed(1)
    emb = torch.randn((300, 64), generator=g).to(DEV)
    qry = torch.randn((2, 64), generator=g).to(DEV)
    idx, sc, uni, cnt = binding.reform_gather_topk(emb, qry, 300, 0)                    # k = N
    torch.cuda.synchronize()
    assert (idx.cpu().numpy() == np.arange(300)[None, :]).all() and int(cnt.item()) == 300
    sim_ref = oracle.cosine(to_np(emb), to_np(qry))
    assert_close(sc.cpu().numpy(), sim_ref, RTOL[torch.float32], "scores of the selected rows")
    idx, sc, uni, cnt = binding.reform_gather_topk(emb, qry, 1, 0)                      # k = 1
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy()[:, 0], sim_ref.argmax(axis=1))
    one = torch.randn((1, 64), generator=g).to(DEV)                                     # a one-row context
    idx, _, uni, cnt = binding.reform_gather_topk(one, qry, 1, 5, 3, 3)
    torch.cuda.synchronize()
    assert idx.cpu().numpy().tolist() == [[0], [0]] and int(cnt.item()) == 1 and int(uni[0].item()) == 0
    sel, pooled = binding.reform_gather_pooled(one, qry, 1, 129, 1, 0)
    torch.cuda.synchronize()
    assert sel.cpu().numpy().tolist() == [0]
    assert_close(pooled.cpu().numpy(), oracle.pool_scores(oracle.cosine(to_np(one), to_np(qry)), 129),
                 RTOL[torch.float32], "pooled score of a one-row context")


def test_calls_with_zero_rows_do_nothing():
    g = torch.Generator().manual_seed(2)
    emb = torch.full((10, 64), 3.0, dtype=torch.bfloat16, device=DEV)
    src = torch.randn((10, 32), generator=g).bfloat16().to(DEV)
    binding.reform_embed_save_selected(src[:0], emb, 0, 32)
    table = torch.randn((10, 64), generator=g).bfloat16().to(DEV)
    out = torch.full((4, 64), 2.0, dtype=torch.bfloat16, device=DEV)
    binding.reform_gather_rows(table, torch.zeros((0,), dtype=torch.int32, device=DEV), out=out)
    zero = torch.zeros((1,), dtype=torch.int32, device=DEV)
    binding.reform_gather_rows(table, torch.arange(4, dtype=torch.int32, device=DEV), count=zero, out=out)
    k = torch.randn((2, 20, 64), generator=g).bfloat16().to(DEV)
    k0 = k.clone()
    kept = torch.arange(8, dtype=torch.int32, device=DEV).repeat(2, 1).contiguous()
    binding.reform_rerotate_keys(k, kept, 0)
    binding.reform_rerotate_keys(k, kept, 8)                                           # nothing moved
    torch.cuda.synchronize()
    assert (emb == 3.0).all() and (out == 2.0).all() and torch.equal(k, k0)


def test_single_query_single_key_attention():
    q = torch.tensor([[[1.0, -2.0, 0.5, 0.25]]], device=DEV)                            # 1 head, 1 row, d = 4
    k = torch.tensor([[[0.5, 0.5, -1.0, 2.0]]], device=DEV)
    v = torch.tensor([[[3.0, -1.0, 0.0, 7.0]]], device=DEV)
    out, lse, score = binding.reform_chunk_attend_score(q, k, v, 0, 0.5)
    torch.cuda.synchronize()
    o_ref, l_ref, s_ref = oracle.attend_score(to_np(q), to_np(k), to_np(v), 0, 0.5)
    assert_close(to_np(out), o_ref, 1e-6, "out")            # the only key has probability 1
    assert_close(to_np(lse), l_ref, 1e-6, "lse")
    assert float(score[0, 0]) == 1.0 and s_ref[0, 0] == 1.0

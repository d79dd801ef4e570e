"""GPU parity of reform_gather_pooled (the selection of Sec. 3.3 in the paper's own order: max over
query tokens, 129-token max-pool, forced first/last tokens, top budget) against the fp64 oracle.

The pooled scores are compared element by element (bf16 tolerance 2e-2, fp32 1e-5).  Pooled
scores form plateaus (a maximum is shared by up to `window` neighbours), so exact ties at the
budget boundary are the normal case: the selection must be exact, lowest index first, on the
GPU's own fp32 pooled scores (checked with numpy), and against the oracle it must agree except
for candidates whose oracle score is within the tolerance of the boundary score.
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import RTOL, assert_close, assert_selection_within_band, stores_for, to_np
from paper_2506_01215_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def exact_on_own_scores(pooled, budget, n_head, n_tail):
    n = pooled.shape[0]
    key = pooled.astype(np.float64).copy()
    key[:n_head] = np.inf
    if n_tail:
        key[n - n_tail:] = np.inf
    return np.sort(np.lexsort((np.arange(n), -key))[:budget])


def check(emb, qry, budget, window, n_head, n_tail, rtol, label, ref=None):
    print(f"[pooled] {label}: N={emb.shape[0]} D={emb.shape[1]} nq={qry.shape[0]} budget={budget} "
          f"window={window} keep={n_head}/{n_tail}", flush=True)
    sel, pooled = binding.reform_gather_pooled(emb, qry, budget, window, n_head, n_tail)
    torch.cuda.synchronize()
    sel_h, pooled_h = sel.cpu().numpy(), pooled.cpu().numpy()
    emb_o, qry_o = ref if ref is not None else (emb, qry)
    _, p_ref, s_ref = oracle.gather_pooled(to_np(emb_o), to_np(qry_o), budget, window, n_head, n_tail)
    assert_close(pooled_h, p_ref, rtol, f"{label}: pooled scores")
    np.testing.assert_array_equal(sel_h, exact_on_own_scores(pooled_h, budget, n_head, n_tail))
    n = emb.shape[0]
    forced = list(range(n_head)) + list(range(n - n_tail, n))
    subs = assert_selection_within_band(sel_h, p_ref, budget, rtol, f"{label}: selection", forced)
    if subs == 0:
        np.testing.assert_array_equal(sel_h, s_ref)
    return subs


@pytest.mark.parametrize("N,D,nq,budget,window,keep", [
    (2048, 256, 1, 128, 129, 0),          # workload-1 shape, one query token
    (5000, 64, 3, 700, 129, 256),         # ragged N (not a multiple of the tile), forced ends
    (3000, 64, 5, 400, 17, 16),           # the ablation's smaller windows (Table 6a)
    (3000, 64, 5, 400, 5, 16),
    (1000, 32, 2, 50, 1, 0),              # window 1: only the max over query tokens
    (700, 32, 4, 700, 129, 256),          # budget = N: everything selected
    (9000, 32, 20, 1200, 1025, 0),        # largest supported window, more than 16 query tokens
])
def test_fp32_small(N, D, nq, budget, window, keep):
    g = torch.Generator(device="cpu").manual_seed(N + window)
    emb = torch.randn((N, D), generator=g).to(DEV)
    qry = torch.randn((nq, D), generator=g).to(DEV)
    check(emb, qry, budget, window, keep, keep, RTOL[torch.float32], f"fp32 N={N} w={window}")


def test_exact_plateau_ties_lowest_index_first():
    """Embeddings drawn from 12 templates: the similarities take 12 values that are far apart, so
    the GPU and the oracle agree on every comparison and the lowest-index rule decides."""
    g = torch.Generator(device="cpu").manual_seed(7)
    D, N = 64, 6000
    templ = torch.randn((12, D), generator=g)
    which = torch.randint(0, 12, (N,), generator=g)
    emb = templ[which].contiguous().to(DEV)
    qry = (templ[3] + 0.5 * templ[8])[None].contiguous().to(DEV)
    for budget in (1, 129, 500, 3000):
        subs = check(emb, qry, budget, 129, 0, 0, RTOL[torch.float32], f"templates budget={budget}")
        assert subs == 0


def test_bf16_workload2_shape_scaled():
    gcfg = synth.GATHERS[2]
    emb, qry = synth.gather_inputs(gcfg, DEV)
    emb = emb[:40000].contiguous()
    qry = torch.cat([qry, emb[12345:12348] + 0.25 * emb[777:780]]).contiguous()     # 4 query tokens
    check(emb, qry, 4096, 129, 256, 256, RTOL[torch.bfloat16], "bf16 40000 x 1024")


def test_bf16_workload4_full_size():
    """N = 1 048 576, D = 2048, 16 query tokens, budget 16384, window 129, 256 + 256 forced:
    the configuration bench.py times for this call."""
    gcfg = synth.GATHERS[4]
    emb, qry, emb_o, qry_o = stores_for(gcfg, *synth.gather_inputs(gcfg, DEV))
    check(emb, qry, 16384, 129, 256, 256, RTOL[torch.bfloat16], "bf16 workload 4", ref=(emb_o, qry_o))

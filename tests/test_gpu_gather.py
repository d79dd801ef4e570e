"""GPU parity: reform_gather_topk against the fp64 CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
from helpers import RTOL, assert_close, assert_selection_within_band, numpy_union, stores_for, to_np
from paper_2506_01215_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_case(emb, qry, k, radius=0, n_head=0, n_tail=0, expect_exact=False, ref=None):
    """ref: (emb, qry) as the oracle side sees them when each side builds its own store."""
    dtype = emb.dtype
    N, D = emb.shape
    nq = qry.shape[0]
    print(f"[gather] {dtype} N={N} D={D} nq={nq} k={k} r={radius} keep={n_head}/{n_tail}", flush=True)
    ed, qd = emb.to(DEV), qry.to(DEV)
    sim = binding.reform_gather_similarity(ed, qd)
    idx, sc, uni, cnt = binding.reform_gather_topk(ed, qd, k, radius, n_head, n_tail)
    torch.cuda.synchronize()
    emb_o, qry_o = ref if ref is not None else (emb, qry)
    sim_ref, topk_ref, uni_ref = oracle.gather(to_np(emb_o), to_np(qry_o), k, radius, n_head, n_tail)
    rtol = RTOL[dtype]
    assert_close(sim.cpu().numpy(), sim_ref, rtol, "sim")
    idx_h, sc_h = idx.cpu().numpy(), sc.cpu().numpy()
    subs = 0
    for q in range(nq):
        subs += assert_selection_within_band(idx_h[q], sim_ref[q], k, rtol, f"topk q={q}")
        # reported scores are the similarities of the reported rows
        np.testing.assert_array_equal(sc_h[q], sim.cpu().numpy()[q, idx_h[q]])
    c = int(cnt.item())
    got_union = uni.cpu().numpy()[:c]
    np.testing.assert_array_equal(got_union, numpy_union(idx_h, N, radius, n_head, n_tail))
    if subs == 0:
        np.testing.assert_array_equal(idx_h, topk_ref)
        np.testing.assert_array_equal(got_union, uni_ref)
    if expect_exact:
        assert subs == 0
    return subs


def test_workload1_fp32_full():
    cfg = synth.GATHERS[1]
    emb, qry = synth.gather_inputs(cfg)
    run_case(emb, qry, cfg.k, cfg.radius)


@pytest.mark.parametrize("N,D,nq,k,r,dtype", [
    (1000, 64, 1, 10, 0, torch.float32),
    (4099, 256, 3, 257, 2, torch.float32),        # N not a multiple of anything
    (5000, 1024, 1, 500, 0, torch.bfloat16),
    (8191, 2048, 16, 300, 8, torch.bfloat16),     # 16 queries, ragged last 16-row group
    (9000, 128, 17, 64, 3, torch.bfloat16),       # two query groups
    (3000, 72, 2, 100, 1, torch.bfloat16),        # dim not a multiple of 32: generic kernel
    (70000, 256, 2, 70000, 0, torch.bfloat16),    # k = N
    (33, 64, 1, 1, 40, torch.bfloat16),           # radius covers everything
])
def test_matches_oracle(N, D, nq, k, r, dtype):
    g = torch.Generator().manual_seed(N + D)
    emb = torch.randn((N, D), generator=g).to(dtype)
    qry = torch.randn((nq, D), generator=g).to(dtype)
    run_case(emb, qry, k, r)


def test_forced_first_and_last_rows():
    g = torch.Generator().manual_seed(4)
    emb = torch.randn((6000, 256), generator=g).bfloat16()
    qry = torch.randn((4, 256), generator=g).bfloat16()
    run_case(emb, qry, 50, 4, n_head=256, n_tail=256)
    run_case(emb, qry, 50, 0, n_head=1, n_tail=7000 - 1000)


@pytest.mark.parametrize("dtype", [torch.float32, torch.bfloat16])
def test_exact_ties_take_the_lowest_index(dtype):
    """Rows drawn from 40 templates with well separated cosines: every similarity value occurs
    many times, the cut falls inside a tie group, and the result must equal the oracle's exactly."""
    g = torch.Generator().manual_seed(8)
    D, N, T = 256, 6000, 40
    u = torch.randn(D, generator=g, dtype=torch.float64)
    u /= u.norm()
    w = torch.randn((T, D), generator=g, dtype=torch.float64)
    w -= (w @ u)[:, None] * u[None, :]
    w /= w.norm(dim=1, keepdim=True)
    c = torch.linspace(-0.9, 0.9, T, dtype=torch.float64)[:, None]
    templates = (c * u[None, :] + torch.sqrt(1 - c * c) * w) * 3.0
    pick = torch.randint(0, T, (N,), generator=g)
    emb = templates[pick].to(dtype)
    qry = (u * 2.0)[None, :].to(dtype)
    for k in (1, 77, 1500, 5999):
        run_case(emb, qry, k, 1, expect_exact=True)


def test_zero_rows_hit_the_eps_clamp():
    g = torch.Generator().manual_seed(10)
    emb = torch.randn((2048, 128), generator=g).bfloat16()
    emb[::7] = 0
    qry = torch.randn((2, 128), generator=g).bfloat16()
    run_case(emb, qry, 100, 0)


def test_normalised_head_embeddings_small():
    cfg = synth.scaled(synth.GATHERS[4], N=20000, k=512)
    emb_d, qry_d, emb_o, qry_o = stores_for(cfg, *synth.gather_inputs(cfg))
    run_case(emb_d, qry_d, cfg.k, cfg.radius, ref=(emb_o, qry_o))

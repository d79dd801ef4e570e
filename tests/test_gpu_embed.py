"""GPU parity of reform_embed_save_selected (Sec. 3.2 normalise-and-concatenate, Alg. 1
SaveSelected) against the fp64 oracle, and the data flow embedding store -> gather."""
import numpy as np
import pytest
import torch

import oracle
from helpers import RTOL, assert_close, assert_selection_within_band, to_np
from paper_2506_01215_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def build_store(states, picks, N, dtype, chunk):
    """states[kind] is [heads][N][d]; picks = list of (kind, head).  Fills the store chunk by chunk
    on the GPU and, independently, with the oracle."""
    d = states[0].shape[2]
    D = d * len(picks)
    emb = torch.zeros((N, D), dtype=dtype, device=DEV)
    ref = np.zeros((N, D))
    dev_states = [s.to(DEV) for s in states]
    for t0 in range(0, N, chunk):
        t1 = min(t0 + chunk, N)
        for seg, (kind, head) in enumerate(picks):
            binding.reform_embed_save_selected(dev_states[kind][head, t0:t1], emb, t0, seg * d)
    for seg, (kind, head) in enumerate(picks):
        oracle.embed_segment(to_np(states[kind][head]), ref, seg * d)
    torch.cuda.synchronize()
    return emb, ref


@pytest.mark.parametrize("dtype,d,N,chunk", [
    (torch.float32, 64, 300, 128),       # fp32, 16 lanes per row
    (torch.float32, 4, 50, 50),          # one 16-byte piece per row
    (torch.bfloat16, 128, 1000, 333),    # the models' head_dim, ragged chunks
    (torch.bfloat16, 64, 257, 64),
    (torch.bfloat16, 8, 70, 70),         # one piece per row
    (torch.bfloat16, 96, 100, 100),      # 12 pieces: group of 16 lanes with 4 idle
    (torch.bfloat16, 512, 40, 40),       # a full wave per row
])
def test_store_matches_oracle(dtype, d, N, chunk):
    g = torch.Generator().manual_seed(d + N)
    q = (torch.randn((3, N, d), generator=g) * 3.0).to(dtype)
    k = torch.randn((2, N, d), generator=g).to(dtype)
    k[1, 5] = 0                                           # a zero vector stays zero
    picks = [(0, 2), (1, 0), (0, 0), (1, 1)]
    print(f"[embed] dtype={dtype} d={d} N={N} chunk={chunk}", flush=True)
    emb, ref = build_store([q, k], picks, N, dtype, chunk)
    got = to_np(emb)
    assert_close(got, ref, RTOL[dtype], "embedding store")
    assert np.all(got[5, 3 * d:4 * d] == 0)
    norms = np.linalg.norm(got.reshape(N, 4, d), axis=2)
    norms[5, 3] = 1.0
    np.testing.assert_allclose(norms, 1.0, rtol=4e-3 if dtype == torch.bfloat16 else 1e-6)


def test_strided_source_rows_and_untouched_columns():
    """The head vector sits inside a [rows][heads][d] tensor; other columns of the store keep
    their content."""
    g = torch.Generator().manual_seed(5)
    n, H, d = 200, 6, 128
    x = torch.randn((n, H, d), generator=g).bfloat16().to(DEV)
    emb = torch.full((n, 4 * d), 2.0, dtype=torch.bfloat16, device=DEV)
    binding.reform_embed_save_selected(x[:, 4], emb, 0, 2 * d)
    torch.cuda.synchronize()
    ref = np.zeros((n, d))
    oracle.embed_segment(to_np(x[:, 4].contiguous()), ref, 0)
    got = to_np(emb)
    assert_close(got[:, 2 * d:3 * d], ref, RTOL[torch.bfloat16], "segment")
    assert np.all(got[:, :2 * d] == 2.0) and np.all(got[:, 3 * d:] == 2.0)


@pytest.mark.parametrize("dtype,d", [(torch.bfloat16, 128), (torch.float32, 64)])
def test_several_heads_in_one_call(dtype, d):
    """Heads 1..4 of a [heads][rows][d] tensor (and of a [rows][heads][d] one) written as four
    adjacent segments by a single call; identical to four one-head calls and to the oracle."""
    g = torch.Generator().manual_seed(11)
    n, H = 777, 6
    x = (torch.randn((H, n, d), generator=g) * 2.0).to(dtype)
    xd = x.to(DEV)
    emb = torch.full((n, 6 * d), 3.0, dtype=dtype, device=DEV)
    binding.reform_embed_save_selected(xd[1:5], emb, 0, d)
    xt = xd.transpose(0, 1).contiguous()                      # [rows][heads][d]
    emb_t = torch.full((n, 6 * d), 3.0, dtype=dtype, device=DEV)
    binding.reform_embed_save_selected(xt.transpose(0, 1)[1:5], emb_t, 0, d)
    emb_1 = torch.full((n, 6 * d), 3.0, dtype=dtype, device=DEV)
    for h in range(1, 5):
        binding.reform_embed_save_selected(xd[h], emb_1, 0, h * d)
    torch.cuda.synchronize()
    ref = np.full((n, 6 * d), 3.0)
    for h in range(1, 5):
        oracle.embed_segment(to_np(x[h]), ref, h * d)
    assert_close(to_np(emb), ref, RTOL[dtype], "four heads, one call")
    assert torch.equal(emb, emb_1) and torch.equal(emb_t, emb_1)


def test_store_feeds_the_gather():
    """Embedding store built on the GPU from 4 layers x 4 heads of synthetic Q/K states, then the
    paper's selection on it; the oracle builds its own store in fp64 and selects from that."""
    g = torch.Generator().manual_seed(9)
    N, d, nq = 20000, 128, 8
    layers = [torch.randn((4, N + nq, d), generator=g).bfloat16() for _ in range(4)]   # last nq tokens = the query
    picks = [(l, h) for l in range(4) for h in range(4)]
    emb_all, ref_all = build_store(layers, picks, N + nq, torch.bfloat16, 4096)
    emb, qry = emb_all[:N].contiguous(), emb_all[N:].contiguous()
    sel, pooled = binding.reform_gather_pooled(emb, qry, 2048, 129, 256, 256)
    torch.cuda.synchronize()
    _, p_ref, s_ref = oracle.gather_pooled(ref_all[:N].astype(np.float32), ref_all[N:].astype(np.float32),
                                           2048, 129, 256, 256)
    assert_close(pooled.cpu().numpy(), p_ref, RTOL[torch.bfloat16], "pooled scores from the GPU-built store")
    forced = list(range(256)) + list(range(N - 256, N))
    assert_selection_within_band(sel.cpu().numpy(), p_ref, 2048, RTOL[torch.bfloat16], "selection", forced)

"""The seeded generators: shapes, determinism and the planted structure (CPU only)."""
import math

import torch

from paper_2506_01215_amd import synth


def test_stream_shapes_and_determinism():
    for cid, cfg in synth.STREAMS.items():
        small = synth.scaled(cfg, L=3 * 64 + 17, C=64, B=32)
        assert small.n_chunks == 4 and small.chunk_len(3) == 17
        q, k, v = synth.chunk_qkv(small, 0, 1)
        q2, k2, v2 = synth.chunk_qkv(small, 0, 1)
        assert q.shape == (cfg.n_q_heads, 64, cfg.head_dim) and q.dtype == cfg.dtype
        assert k.shape == v.shape == (cfg.n_kv_heads, 64, cfg.head_dim)
        assert torch.equal(q, q2) and torch.equal(k, k2) and torch.equal(v, v2)
        q3, _, _ = synth.chunk_qkv(small, 0, 2)
        assert not torch.equal(q, q3)
        assert synth.chunk_qkv(small, 0, 3)[0].shape[1] == 17


def test_lowrank_basis_is_orthonormal_and_unit_variance():
    cfg = synth.scaled(synth.STREAMS[3], L=4096, C=4096, B=64)
    U = synth.lowrank_basis(cfg, 5, "cpu")
    assert torch.allclose(U @ U.t(), torch.eye(16), atol=1e-5)
    q, k, _ = synth.chunk_qkv(cfg, 5, 0)
    assert abs(q.float().var().item() - 1.0) < 0.05 and abs(k.float().var().item() - 1.0) < 0.05


def test_adversarial_structure():
    cfg = synth.scaled(synth.STREAMS[5], L=2048 + 17, C=512, B=128)
    plan = synth.adversarial_plan(cfg)
    q, k, v = synth.chunk_qkv(cfg, 0, 0, plan=plan)
    u = plan["u"]
    d = cfg.head_dim
    # sinks: tokens 0..3 have key norm 8*sqrt(d) along u
    assert torch.allclose(k[:, :4].float().norm(dim=-1), torch.full((8, 4), 8 * math.sqrt(d)), rtol=1e-2)
    # exact duplicates exist among the keys of a chunk
    rows = k[0].view(torch.int16)
    uniq = torch.unique(rows, dim=0).shape[0]
    assert uniq < rows.shape[0] - 10
    assert cfg.chunk_len(cfg.n_chunks - 1) == 17
    assert (plan["needle_pos"] >= 4).all() and (plan["needle_pos"] < cfg.L).all()
    cos = torch.nn.functional.cosine_similarity(q[:, 100].float(), u, dim=-1)
    assert (cos > 0).all()


def test_gather_inputs():
    cfg = synth.scaled(synth.GATHERS[4], N=300, n_query=3, k=16)
    emb, qry = synth.gather_inputs(cfg, block_rows=128)
    assert emb.shape == (300, 2048) and qry.shape == (3, 2048) and emb.dtype == torch.bfloat16
    # raw head states: the per-head normalisation is the embedding-construction step's job, not the generator's
    seg = emb.float().view(300, 16, 128).norm(dim=-1)
    assert (seg - 128 ** 0.5).abs().mean() < 1.0 and seg.std() > 0.3
    assert synth.GATHERS[4].kind == "head_states"
    emb2, _ = synth.gather_inputs(cfg, block_rows=128)
    assert torch.equal(emb, emb2)

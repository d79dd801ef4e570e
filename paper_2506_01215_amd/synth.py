"""Seeded synthetic inputs shaped like the paper's long-context workloads.

This module only draws random tensors.  It contains none of the method's
arithmetic (no attention, no scoring, no selection, no similarity) and loads
no native code, so both the GPU tests/benchmark and the CPU oracle's tests can
use it.  The paper runs public long-context suites through pretrained models
(Sec. 4); neither is available offline, so these generators reproduce only the
shapes and the statistical structure: 32k-token chunks with a 32k cache budget
(Sec. 3.1, Sec. 4 setup), GQA 32/8 x 128 layers, 8k-16k gather budgets, and
embeddings made of four selected heads (App. C.6).

Five workloads are defined (ids 1..5); `STREAMS[id]` describes the recurrent
chunked stream, `GATHERS[id]` the gather problem.  All draws are functions of
(seed, layer, chunk index), so any chunk can be regenerated on its own.
"""
from dataclasses import dataclass, replace
import math

import torch


@dataclass(frozen=True)
class StreamConfig:
    name: str
    kind: str            # iid | lognormal_knorm | lowrank | adversarial
    dtype: torch.dtype
    n_layers: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    L: int               # context length
    C: int               # chunk length
    B: int               # cache budget per KV head
    seed: int = 0

    @property
    def n_chunks(self):
        return (self.L + self.C - 1) // self.C

    def chunk_len(self, t):
        return min(self.C, self.L - t * self.C)

    @property
    def scale(self):
        return 1.0 / math.sqrt(self.head_dim)

    @property
    def capacity(self):
        return self.B + self.C


@dataclass(frozen=True)
class GatherConfig:
    name: str
    kind: str            # iid | head_states (rows are the concatenated raw states of D/128 heads)
    dtype: torch.dtype
    N: int
    D: int
    n_query: int
    k: int
    radius: int = 0
    seed: int = 0


STREAMS = {
    1: StreamConfig("cfg1_tiny_fp32", "iid", torch.float32, 1, 4, 4, 64, 2048, 128, 256, 0),
    2: StreamConfig("cfg2_llama3_8b_layer_128k", "lognormal_knorm", torch.bfloat16, 1, 32, 8, 128,
                    131072, 8192, 8192, 2),
    3: StreamConfig("cfg3_mistral7b_1m", "lowrank", torch.bfloat16, 32, 32, 8, 128,
                    1048576, 32768, 32768, 3),
    5: StreamConfig("cfg5_adversarial_ragged", "adversarial", torch.bfloat16, 1, 8, 8, 128,
                    1048593, 16384, 4096, 5),
}

GATHERS = {
    1: GatherConfig("cfg1_gather_fp32", "iid", torch.float32, 2048, 256, 1, 128, 0, 0),
    2: GatherConfig("cfg2_gather_128k", "iid", torch.bfloat16, 131072, 1024, 1, 4096, 0, 2),
    4: GatherConfig("cfg4_gather_1m", "head_states", torch.bfloat16, 1048576, 2048, 16, 16384,
                    8, 4),
}


def scaled(cfg, **kw):
    """A copy of a config with some sizes replaced (small versions for CPU-timed checks)."""
    return replace(cfg, **kw)


def _gen(device, *key):
    """torch.Generator seeded from an integer tuple (splitmix-style mixing, host side)."""
    x = 0x9E3779B97F4A7C15
    for v in key:
        x = (x ^ (int(v) + 0x9E3779B97F4A7C15 + ((x << 6) & 0xFFFFFFFFFFFFFFFF) + (x >> 2))) \
            & 0xFFFFFFFFFFFFFFFF
        x = (x * 0xBF58476D1CE4E5B9) & 0xFFFFFFFFFFFFFFFF
        x ^= x >> 31
    g = torch.Generator(device=device)
    g.manual_seed(x & 0x7FFFFFFFFFFFFFFF)
    return g


def _randn(shape, g, device):
    return torch.randn(shape, generator=g, device=device, dtype=torch.float32)


def _unit(x):
    return x / x.norm(dim=-1, keepdim=True)


def lowrank_basis(cfg, layer, device):
    """16 x d row-orthonormal basis shared by the Q and K of one layer (workload 3)."""
    g = _gen("cpu", cfg.seed, 101, layer)
    a = torch.randn((cfg.head_dim, 16), generator=g, dtype=torch.float64)
    qmat, _ = torch.linalg.qr(a)          # d x 16, orthonormal columns
    return qmat.t().contiguous().to(torch.float32).to(device)


def adversarial_plan(cfg):
    """Fixed planted structure of workload 5 (host tensors, fp32)."""
    H, d = cfg.n_kv_heads, cfg.head_dim
    g = _gen("cpu", cfg.seed, 202)
    u = _unit(torch.randn((H, d), generator=g))                  # sink / bias direction per head
    w = _unit(torch.randn((H, 64, d), generator=g))              # needle directions
    templates = torch.randn((H, 256, d), generator=g)            # duplicated-key templates
    lo = min(4, cfg.L - 1)
    needle_pos = torch.randperm(max(cfg.L - lo, 1), generator=g)[:64] + lo
    return {"u": u, "w": w, "templates": templates, "needle_pos": needle_pos.sort().values}


def chunk_qkv(cfg, layer, t, device="cpu", plan=None, basis=None):
    """Q [Hq,Ct,d], K [Hkv,Ct,d], V [Hkv,Ct,d] of chunk t of one layer, in cfg.dtype."""
    Ct = cfg.chunk_len(t)
    Hq, Hkv, d = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim
    g = _gen(device, cfg.seed, 7, layer, t)
    q = _randn((Hq, Ct, d), g, device)
    k = _randn((Hkv, Ct, d), g, device)
    v = _randn((Hkv, Ct, d), g, device)
    if cfg.kind == "iid":
        pass
    elif cfg.kind == "lognormal_knorm":
        # per-token key norm ~ LogNormal(0, 0.5), one scalar per token shared by the KV heads
        z = _randn((1, Ct, 1), _gen(device, cfg.seed, 8, t), device)
        k = k * torch.exp(0.5 * z)
    elif cfg.kind == "lowrank":
        rho = 0.5
        U = basis if basis is not None else lowrank_basis(cfg, layer, device)
        z = _randn((Ct, 16), _gen(device, cfg.seed, 9, t), device)     # shared by q and k of a token
        shared = (z @ U) * math.sqrt(rho * d / 16.0)                   # [Ct, d]
        q = math.sqrt(1.0 - rho) * q + shared.unsqueeze(0)
        k = math.sqrt(1.0 - rho) * k + shared.unsqueeze(0)
    elif cfg.kind == "adversarial":
        assert Hq == Hkv
        plan = plan if plan is not None else adversarial_plan(cfg)
        u = plan["u"].to(device)
        w = plan["w"].to(device)
        tm = plan["templates"].to(device)
        base = t * cfg.C
        q = q + 2.0 * u.unsqueeze(1)
        # 25 % of tokens copy their key bit-for-bit from one of 256 templates
        gd = _gen(device, cfg.seed, 10, t)
        is_dup = torch.rand((Ct,), generator=gd, device=device) < 0.25
        tid = torch.randint(0, 256, (Ct,), generator=gd, device=device)
        k = torch.where(is_dup.view(1, Ct, 1), tm[:, tid, :], k)
        # every chunk carries one probe query per needle direction
        rows = (torch.arange(64, device=device) * cfg.C // 64 + 7) % Ct
        eps = _randn((Hq, 64, d), gd, device)
        q[:, rows, :] = 6.0 * w + eps
        # needle keys at their global positions, sinks at tokens 0..3
        npos = plan["needle_pos"].to(device)
        inside = (npos >= base) & (npos < base + Ct)
        if bool(inside.any()):
            k[:, (npos[inside] - base), :] = 3.0 * math.sqrt(d) * w[:, inside, :]
        if base == 0:
            ns = min(4, Ct)
            k[:, :ns, :] = (8.0 * math.sqrt(d)) * u.unsqueeze(1).expand(Hkv, ns, d)
    else:
        raise ValueError(cfg.kind)
    return q.to(cfg.dtype), k.to(cfg.dtype), v.to(cfg.dtype)


def gather_inputs(cfg, device="cpu", block_rows=65536):
    """emb [N,D], qry [nq,D] in cfg.dtype.

    kind "iid": the rows are the embeddings themselves.  kind "head_states": the rows are the raw
    N(0,1) states of D/128 selected (layer, head) pairs side by side; the embedding store of that
    workload is what the embedding-construction step makes of them (Sec. 3.2 equation: every head
    segment L2-normalised).  That step is the method's arithmetic and is not done here: the GPU
    side builds its store with the library call, the oracle side with the oracle's own routine."""
    if cfg.kind not in ("iid", "head_states"):
        raise ValueError(cfg.kind)
    if cfg.kind == "head_states":
        assert cfg.D % 128 == 0

    def draw(rows, g):
        return _randn((rows, cfg.D), g, device).to(cfg.dtype)

    emb = torch.empty((cfg.N, cfg.D), dtype=cfg.dtype, device=device)
    for b, r0 in enumerate(range(0, cfg.N, block_rows)):
        r1 = min(cfg.N, r0 + block_rows)
        emb[r0:r1] = draw(r1 - r0, _gen(device, cfg.seed, 11, b))
    qry = draw(cfg.n_query, _gen(device, cfg.seed, 12))
    return emb, qry

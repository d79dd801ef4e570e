"""The library calls under HIP graph capture and on concurrent streams: every call only enqueues
kernels on the stream it is given (no allocation, no synchronisation, no memset nodes, no state
kept between calls), so a layer-step and a gather can be captured once and replayed, and two
streams can run the library at the same time.  Each replay is checked against the eager result
on the same inputs, with eager work and synchronisations between the replays."""
import pytest
import torch

from paper_2506_01215_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def test_layer_step_replays_match_eager():
    Hq, Hkv, d, C, B = 8, 2, 128, 1024, 1024
    M, cap = B, B + C
    scale = d ** -0.5
    g = torch.Generator(device=DEV).manual_seed(21)
    rnd = lambda *s: torch.randn(s, generator=g, device=DEV).bfloat16()
    K0, V0 = rnd(Hkv, cap, d), rnd(Hkv, cap, d)
    pos0 = torch.arange(cap, dtype=torch.int32, device=DEV).repeat(Hkv, 1).contiguous()
    qs = [rnd(Hq, C, d) for _ in range(3)]

    def buffers():
        return dict(q=torch.empty_like(qs[0]), K=torch.empty_like(K0), V=torch.empty_like(V0),
                    pos=torch.empty_like(pos0), out=torch.empty_like(qs[0]),
                    lse=torch.empty((Hq, C), dtype=torch.float32, device=DEV),
                    score=torch.empty((Hkv, cap), dtype=torch.float32, device=DEV),
                    kept=torch.empty((Hkv, B), dtype=torch.int32, device=DEV),
                    wsa=torch.empty(binding.attend_workspace_bytes(
                        binding.attn_desc(qs[0], K0, qs[0], M, scale)) + 512, dtype=torch.uint8, device=DEV),
                    wse=torch.empty(binding.evict_workspace_bytes(binding.evict_desc(K0, M + C, B, 4, 4)) + 512,
                                    dtype=torch.uint8, device=DEV))

    def step(b):
        b["K"].copy_(K0)
        b["V"].copy_(V0)
        b["pos"].copy_(pos0)
        binding.reform_chunk_attend_score(b["q"], b["K"], b["V"], M, scale, out=b["out"], lse=b["lse"],
                                          score=b["score"], workspace=b["wsa"])
        binding.reform_evict_topk_compact(b["K"], b["V"], b["score"], M + C, B, 4, 4, pos=b["pos"],
                                          kept_idx=b["kept"], workspace=b["wse"])
        binding.reform_rerotate_keys(b["K"], b["kept"], B, theta=1e6)

    eager, graphed = buffers(), buffers()
    graphed["q"].copy_(qs[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(graphed)                                     # warm-up outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(graphed)
    for r, q in enumerate(qs):
        print(f"[graph] layer-step replay {r}", flush=True)
        eager["q"].copy_(q)
        step(eager)
        torch.cuda.synchronize()
        graphed["q"].copy_(q)
        graph.replay()
        torch.cuda.synchronize()
        for name in ("out", "lse", "score", "kept", "pos"):
            assert torch.equal(eager[name][..., :B] if name in ("score", "pos") else eager[name],
                               graphed[name][..., :B] if name in ("score", "pos") else graphed[name]), name
        assert torch.equal(eager["K"][:, :B], graphed["K"][:, :B])
        assert torch.equal(eager["V"][:, :B], graphed["V"][:, :B])


def test_gather_replays_match_eager():
    N, D, nq, k, r = 70000, 256, 5, 900, 3
    g = torch.Generator(device=DEV).manual_seed(22)
    embs = [torch.randn((N, D), generator=g, device=DEV).bfloat16() for _ in range(3)]
    qry = torch.randn((nq, D), generator=g, device=DEV).bfloat16()
    desc = binding.gather_desc(embs[0], qry, k, r, 7, 9)

    def buffers():
        return dict(emb=torch.empty_like(embs[0]),
                    ti=torch.empty((nq, k), dtype=torch.int32, device=DEV),
                    ts=torch.empty((nq, k), dtype=torch.float32, device=DEV),
                    ui=torch.empty((N,), dtype=torch.int32, device=DEV),
                    uc=torch.zeros((1,), dtype=torch.int32, device=DEV),
                    ws=torch.empty(binding.gather_workspace_bytes(desc) + 512, dtype=torch.uint8, device=DEV))

    def run(b):
        binding.reform_gather_topk(b["emb"], qry, k, r, 7, 9, topk_idx=b["ti"], topk_score=b["ts"],
                                   union_idx=b["ui"], union_count=b["uc"], workspace=b["ws"])

    eager, graphed = buffers(), buffers()
    graphed["emb"].copy_(embs[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run(graphed)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        run(graphed)
    for rep, e in enumerate(embs):
        print(f"[graph] gather replay {rep}", flush=True)
        eager["emb"].copy_(e)
        run(eager)
        torch.cuda.synchronize()
        graphed["emb"].copy_(e)
        graph.replay()
        torch.cuda.synchronize()
        n = int(eager["uc"].item())
        assert n == int(graphed["uc"].item()) and n > 0
        assert torch.equal(eager["ti"], graphed["ti"]) and torch.equal(eager["ts"], graphed["ts"])
        assert torch.equal(eager["ui"][:n], graphed["ui"][:n])


def test_two_streams_with_their_own_workspaces_do_not_interfere():
    """The library keeps no state between calls: two layer-steps issued on two streams at the
    same time, each with its own buffers, give what each gives alone."""
    Hq, Hkv, d, C, B = 8, 2, 128, 2048, 2048
    M, cap = B, B + C
    scale = d ** -0.5
    g = torch.Generator(device=DEV).manual_seed(31)
    rnd = lambda *s: torch.randn(s, generator=g, device=DEV).bfloat16()

    def make():
        b = dict(q=rnd(Hq, C, d), K=rnd(Hkv, cap, d), V=rnd(Hkv, cap, d),
                 pos=torch.arange(cap, dtype=torch.int32, device=DEV).repeat(Hkv, 1).contiguous(),
                 out=torch.empty((Hq, C, d), dtype=torch.bfloat16, device=DEV),
                 lse=torch.empty((Hq, C), dtype=torch.float32, device=DEV),
                 score=torch.empty((Hkv, cap), dtype=torch.float32, device=DEV),
                 kept=torch.empty((Hkv, B), dtype=torch.int32, device=DEV))
        b["wsa"] = torch.empty(binding.attend_workspace_bytes(binding.attn_desc(b["q"], b["K"], b["q"], M, scale)) + 512,
                               dtype=torch.uint8, device=DEV)
        b["wse"] = torch.empty(binding.evict_workspace_bytes(binding.evict_desc(b["K"], M + C, B)) + 512,
                               dtype=torch.uint8, device=DEV)
        return b

    def step(b):
        binding.reform_chunk_attend_score(b["q"], b["K"], b["V"], M, scale, out=b["out"], lse=b["lse"],
                                          score=b["score"], workspace=b["wsa"])
        binding.reform_evict_topk_compact(b["K"], b["V"], b["score"], M + C, B, pos=b["pos"],
                                          kept_idx=b["kept"], workspace=b["wse"])

    jobs = [make() for _ in range(2)]
    alone = []
    for b in jobs:                                        # reference: one after the other
        ref = {k: v.clone() for k, v in b.items()}
        step(ref)
        alone.append(ref)
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(3):                                  # interleaved issue on two streams
        work = [{k: v.clone() for k, v in b.items()} for b in jobs]
        torch.cuda.synchronize()
        for b, st in zip(work, streams):
            with torch.cuda.stream(st):
                step(b)
        torch.cuda.synchronize()
        for b, ref in zip(work, alone):
            for name in ("out", "lse", "kept"):
                assert torch.equal(b[name], ref[name]), (rep, name)
            for name in ("K", "V"):
                assert torch.equal(b[name][:, :B], ref[name][:, :B]), (rep, name)
            assert torch.equal(b["score"][:, :B], ref["score"][:, :B]) and torch.equal(b["pos"][:, :B], ref["pos"][:, :B])


def test_long_row_eviction_under_graph_replay_and_on_two_streams():
    """Eviction at 65536 candidates per head uses several workgroups per row that wait for each
    other inside one launch: captured and replayed on new scores, and issued on two streams at
    once (2 x 128 workgroups fit on the chip together), it gives what the eager call gives, and
    the device-side status word stays clear."""
    Hkv, d, n, B = 8, 64, 65536, 32768
    g = torch.Generator(device=DEV).manual_seed(41)
    K0 = torch.randn((Hkv, n, d), generator=g, device=DEV).bfloat16()
    V0 = torch.randn((Hkv, n, d), generator=g, device=DEV).bfloat16()
    pos0 = torch.arange(n, dtype=torch.int32, device=DEV).repeat(Hkv, 1).contiguous()
    scores = [torch.randint(0, 4096, (Hkv, n), generator=g, device=DEV).float() / 64.0 for _ in range(3)]   # many exact ties
    nws = binding.evict_workspace_bytes(binding.evict_desc(K0, n, B, 4, 4)) + 512

    def buffers():
        return dict(K=torch.empty_like(K0), V=torch.empty_like(V0), pos=torch.empty_like(pos0),
                    s_in=torch.empty_like(scores[0]), score=torch.empty_like(scores[0]),
                    kept=torch.empty((Hkv, B), dtype=torch.int32, device=DEV),
                    ws=torch.full((nws,), 0x5a, dtype=torch.uint8, device=DEV))

    def step(b):
        b["K"].copy_(K0)
        b["V"].copy_(V0)
        b["pos"].copy_(pos0)
        b["score"].copy_(b["s_in"])
        binding.reform_evict_topk_compact(b["K"], b["V"], b["score"], n, B, 4, 4, pos=b["pos"],
                                          kept_idx=b["kept"], workspace=b["ws"])

    def same(a, b):
        assert torch.equal(a["kept"], b["kept"])
        for name in ("K", "V", "score", "pos"):
            assert torch.equal(a[name][:, :B], b[name][:, :B]), name
        assert binding.evict_status_word(a["ws"]) == 0 and binding.evict_status_word(b["ws"]) == 0

    eager, graphed = buffers(), buffers()
    graphed["s_in"].copy_(scores[0])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(graphed)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        step(graphed)
    for r, s in enumerate(scores):
        print(f"[graph] long-row eviction replay {r}", flush=True)
        eager["s_in"].copy_(s)
        step(eager)
        torch.cuda.synchronize()
        graphed["s_in"].copy_(s)
        graph.replay()
        torch.cuda.synchronize()
        same(eager, graphed)
    # two streams at once, each with its own buffers and workspace
    a, b = buffers(), buffers()
    a["s_in"].copy_(scores[1])
    b["s_in"].copy_(scores[2])
    refs = []
    for x, s in ((a, scores[1]), (b, scores[2])):
        eager["s_in"].copy_(s)
        step(eager)
        torch.cuda.synchronize()
        refs.append({k: v.clone() for k, v in eager.items()})
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(3):
        print(f"[graph] long-row eviction on two streams, round {rep}", flush=True)
        torch.cuda.synchronize()
        for x, st in zip((a, b), streams):
            with torch.cuda.stream(st):
                step(x)
        torch.cuda.synchronize()
        same(a, refs[0])
        same(b, refs[1])

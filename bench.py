#!/usr/bin/env python3
"""Benchmark of the REFORM compress-and-gather hot path on one MI355X.

A step = one steady-state chunk of the 1M-token workload (C = B = 32768 tokens, cache full)
pushed through all 32 layers: per layer  reform_chunk_attend_score  (attention over
[cache || chunk] + eviction score) and  reform_evict_topk_compact  (top-B + compaction).  The
cache is first filled by an untimed chunk 0; inputs of every timed step are generated before the
timed region and sit in HBM.  After the timed steps the 1M-row gather (reform_gather_topk,
16 queries, k = 16384, radius 8) is timed on its own and reported as gather_ms.

Prints ONE JSON line.  value = context tokens/s through chunk-compress (steps * C / time).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0         # MI355X HBM3E
# HBM bytes one attn_fwd_bf16 launch of the default workload moves, from the two rocprofv3 --pmc
# runs summarised in profiles/attn_fwd_cfg3_hbm_traffic.md (FETCH_SIZE and WRITE_SIZE in KiB per
# dispatch, each scaled by what the same counter reads for a 1 GiB copy kernel: x2.000 and x1.000).
FWD_TRAFFIC_BYTES = (1737900 * 2.000 + 266240 * 1.000) * 1024


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--layers", type=int, default=0, help="debug only: fewer layers (marks the result invalid)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-gather", action="store_true")
    ap.add_argument("--zero-data", action="store_true",
                    help="debug only: all-zero Q/K/V (marks the result invalid); shows how much of the "
                         "kernel time is the power-limited clock that random operands cause")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the timed region, run a plain 1 GiB -> 1 GiB elementwise copy kernel; "
                         "used to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings to bytes")
    return ap.parse_args()


def cpu_baseline(cfg, q_mid, K, V, M):
    """The fp64 oracle, as it stands, on a bounded sample of the same layer-step: the middle
    rows of the chunk (their cost is the chunk's average), all heads, against the full
    [cache || chunk] key set, plus the per-head selection.  Extrapolated to 32 layers."""
    import numpy as np
    import oracle
    rows = q_mid.shape[1]
    t0 = time.perf_counter()
    _, _, score = oracle.attend_score(q_mid, K, V, M, cfg.scale, want_out=True)
    for g in range(K.shape[0]):
        oracle.evict_select(score[g], M + rows, cfg.B)
    dt = time.perf_counter() - t0
    tok_s = rows / (dt * cfg.n_layers)
    return {"value": tok_s, "unit": "tokens/s", "cores": min(oracle.num_threads(), K.shape[0]),
            "kind": "oracle",
            "sample": f"rows [C/2-{rows // 2}, C/2+{rows // 2}) of one layer-step (32 q heads, "
                      f"{M + rows} keys) + top-B selection, {dt:.1f} s; extrapolated to {cfg.n_layers} layers"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no sharding, no collectives); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2506_01215_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    binding.load_library()
    cfg = synth.STREAMS[3]
    layers = args.layers if args.layers > 0 else cfg.n_layers
    Hq, Hkv, d, C, B = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.C, cfg.B
    cap = cfg.capacity
    K_steps, W_steps = args.steps, args.warmup
    pool = min(K_steps + W_steps, 4)          # distinct pre-generated chunks (cycled beyond that)

    # ---- device buffers (torch = allocator only)
    Kc = [torch.empty((Hkv, cap, d), dtype=cfg.dtype, device=dev) for _ in range(layers)]
    Vc = [torch.empty((Hkv, cap, d), dtype=cfg.dtype, device=dev) for _ in range(layers)]
    score = torch.zeros((Hkv, cap), dtype=torch.float32, device=dev)
    pos = [torch.zeros((Hkv, cap), dtype=torch.int32, device=dev) for _ in range(layers)]
    out = torch.empty((Hq, C, d), dtype=cfg.dtype, device=dev)
    lse = torch.empty((Hq, C), dtype=torch.float32, device=dev)
    kept = torch.empty((Hkv, B), dtype=torch.int32, device=dev)
    ed = binding.evict_desc(Kc[0], B + C, B)
    ws_evict = torch.empty(binding.evict_workspace_bytes(ed) + 256, dtype=torch.uint8, device=dev)
    ws_attn = torch.empty(Hq * C * 4 + 512, dtype=torch.uint8, device=dev)
    bases = [synth.lowrank_basis(cfg, l, dev) for l in range(layers)]

    def gen(t):
        data = [synth.chunk_qkv(cfg, l, t, dev, basis=bases[l]) for l in range(layers)]
        if args.zero_data:
            for qkv in data:
                for x in qkv:
                    x.zero_()
        return data

    # ---- untimed fill: chunk 0 with an empty cache
    tok0 = torch.arange(C, dtype=torch.int32, device=dev)
    for l, (q, k, v) in enumerate(gen(0)):
        Kc[l][:, :C] = k
        Vc[l][:, :C] = v
        pos[l][:, :C] = tok0
        binding.reform_chunk_attend_score(q, Kc[l], Vc[l], 0, cfg.scale, out=out, lse=lse, score=score,
                                          workspace=ws_attn)
        binding.reform_evict_topk_compact(Kc[l], Vc[l], score, C, B, pos=pos[l], kept_idx=kept,
                                          workspace=ws_evict)
    M = min(C, B)
    torch.cuda.synchronize()
    inputs = [gen(1 + s) for s in range(pool)]
    torch.cuda.synchronize()

    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []                                 # (e0, e1, e2, e3) per timed layer-step

    mode = {"obs_window": 0, "n_sink": 0, "n_recent": 0, "rope": False}   # default workload: W = C, nothing forced

    def step(s, timed):
        data = inputs[s % pool]
        W, ns, nr = mode["obs_window"], mode["n_sink"], mode["n_recent"]
        tok = torch.arange((1 + s) * C, (2 + s) * C, dtype=torch.int32, device=dev)
        for l in range(layers):
            q, k, v = data[l]
            for h in range(Hkv):               # the chunk's K/V land at rows [M, M+C) (in a model:
                Kc[l][h, M:M + C].copy_(k[h])  # written there by the QKV projection); per head the
                Vc[l][h, M:M + C].copy_(v[h])  # copy is contiguous (one strided copy_ runs at 0.9 TB/s)
            pos[l][:, M:M + C] = tok
            if timed:
                e = [ev() for _ in range(5)]
                e[0].record()
                binding.reform_chunk_attend_score(q, Kc[l], Vc[l], M, cfg.scale, obs_window=W, out=out,
                                                  lse=lse, score=score, workspace=ws_attn, phases=1)
                e[1].record()
                binding.reform_chunk_attend_score(q, Kc[l], Vc[l], M, cfg.scale, obs_window=W, out=out,
                                                  lse=lse, score=score, workspace=ws_attn, phases=2)
                e[2].record()
                binding.reform_evict_topk_compact(Kc[l], Vc[l], score, M + C, B, ns, nr, pos=pos[l],
                                                  kept_idx=kept, workspace=ws_evict)
                e[3].record()
                if mode["rope"]:
                    binding.reform_rerotate_keys(Kc[l], kept, B, 1e6)
                e[4].record()
                marks.append(e)
            else:
                binding.reform_chunk_attend_score(q, Kc[l], Vc[l], M, cfg.scale, obs_window=W, out=out,
                                                  lse=lse, score=score, workspace=ws_attn)
                binding.reform_evict_topk_compact(Kc[l], Vc[l], score, M + C, B, ns, nr, pos=pos[l],
                                                  kept_idx=kept, workspace=ws_evict)
                if mode["rope"]:
                    binding.reform_rerotate_keys(Kc[l], kept, B, 1e6)

    for s in range(W_steps):
        step(s, False)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for s in range(W_steps, W_steps + K_steps):
        step(s, True)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    ms_step = wall * 1e3 / K_steps
    tok_s = K_steps * C / wall
    fwd_ms = sum(e[0].elapsed_time(e[1]) for e in marks) / len(marks)
    sc_ms = sum(e[1].elapsed_time(e[2]) for e in marks) / len(marks)
    evict_ms = sum(e[2].elapsed_time(e[3]) for e in marks) / len(marks)

    pairs = float(C) * M + C * (C + 1) / 2.0
    fwd_flop = 4.0 * d * pairs * Hq            # QK^T + PV on unmasked pairs
    sc_flop = 2.0 * d * pairs * Hq             # second QK^T of the exact score (executed, not useful)
    elt = 2
    evict_bytes = Hkv * (M + C) * 4.0 + 2.0 * Hkv * B * d * elt * 2    # scores read + K,V rows read+written
    roof = {"kernel": "attn_fwd_bf16", "bound": "mfma", "achieved": fwd_flop / (fwd_ms * 1e-3) / 1e12,
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "traffic": FWD_TRAFFIC_BYTES}
    roof["frac"] = roof["achieved"] / roof["peak"]
    kernels = {
        "attn_fwd_bf16": {"ms": fwd_ms, "tflops": roof["achieved"], "frac_mfma": roof["frac"]},
        "attn_score_bf16": {"ms": sc_ms, "tflops_executed": sc_flop / (sc_ms * 1e-3) / 1e12,
                            "frac_mfma": sc_flop / (sc_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
        "attend_call": {"ms": fwd_ms + sc_ms,
                        "tflops_useful": fwd_flop / ((fwd_ms + sc_ms) * 1e-3) / 1e12,
                        "tflops_executed": (fwd_flop + sc_flop) / ((fwd_ms + sc_ms) * 1e-3) / 1e12},
        "evict_call": {"ms": evict_ms, "gbs": evict_bytes / (evict_ms * 1e-3) / 1e9,
                       "frac_hbm": evict_bytes / (evict_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
    }

    # ---- the same step as the paper's experiments configure the compressor (Sec. 4 common setup:
    # only the last 128 queries of a chunk observe, first and most recent 256 tokens always kept);
    # reported beside the headline figure, never instead of it
    n_main = len(marks)
    mode.update(obs_window=128, n_sink=256, n_recent=256, rope=True)
    step(W_steps + K_steps, False)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    step(W_steps + K_steps + 1, True)
    torch.cuda.synchronize()
    wall_pm = time.perf_counter() - t1
    pm = marks[n_main:]
    paper_mode = {"config": "obs_window 128, n_sink 256, n_recent 256, keys re-rotated to consecutive "
                            "positions (theta 1e6)", "tokens_per_s": C / wall_pm,
                  "ms_per_step": wall_pm * 1e3,
                  "attn_fwd_ms": sum(e[0].elapsed_time(e[1]) for e in pm) / len(pm),
                  "attn_score_ms": sum(e[1].elapsed_time(e[2]) for e in pm) / len(pm),
                  "evict_ms": sum(e[2].elapsed_time(e[3]) for e in pm) / len(pm),
                  "rerotate_ms": sum(e[3].elapsed_time(e[4]) for e in pm) / len(pm)}
    marks = marks[:n_main]

    if args.copy_probe:
        src = torch.ones((1 << 28,), dtype=torch.int32, device=dev)     # 1 GiB read, 1 GiB written
        dst = torch.empty_like(src)
        for _ in range(2):
            torch.add(src, 1, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # ---- CPU baseline sample (oracle), before the gather buffers are allocated
    cpu = None
    if not args.no_cpu_baseline:
        to_np = lambda t: t.detach().float().cpu().numpy()
        q, k, v = inputs[0][0]
        half = 512
        rows = slice(C // 2 - half, C // 2 + half)
        Mo = M + C // 2 - half
        Kh = torch.cat([Kc[0][:, :M], k[:, :C // 2 + half]], dim=1)
        Vh = torch.cat([Vc[0][:, :M], v[:, :C // 2 + half]], dim=1)
        cpu = cpu_baseline(cfg, to_np(q[:, rows]), to_np(Kh), to_np(Vh), Mo)
        del Kh, Vh

    # ---- gather at 1M rows
    gather = None
    if not args.no_gather:
        del inputs
        torch.cuda.empty_cache()
        gcfg = synth.GATHERS[4]
        emb, qry = synth.gather_inputs(gcfg, dev)
        N = gcfg.N
        gd = binding.gather_desc(emb, qry, gcfg.k, gcfg.radius)
        ws = torch.empty(binding.gather_workspace_bytes(gd) + 256, dtype=torch.uint8, device=dev)
        ti = torch.empty((gcfg.n_query, gcfg.k), dtype=torch.int32, device=dev)
        ts = torch.empty((gcfg.n_query, gcfg.k), dtype=torch.float32, device=dev)
        ui = torch.empty((N,), dtype=torch.int32, device=dev)
        uc = torch.zeros((1,), dtype=torch.int32, device=dev)
        sim = torch.empty((gcfg.n_query, N), dtype=torch.float32, device=dev)
        times, sim_times = [], []
        for r in range(7):
            a, b = ev(), ev()
            a.record()
            binding.reform_gather_topk(emb, qry, gcfg.k, gcfg.radius, topk_idx=ti, topk_score=ts,
                                       union_idx=ui, union_count=uc, workspace=ws)
            b.record()
            torch.cuda.synchronize()
            if r >= 2:
                times.append(a.elapsed_time(b))
        for r in range(5):
            a, b = ev(), ev()
            a.record()
            binding.reform_gather_similarity(emb, qry, sim=sim)
            b.record()
            torch.cuda.synchronize()
            if r >= 2:
                sim_times.append(a.elapsed_time(b))
        # the same store through the paper's own post-processing (max over query tokens, 129-token
        # max-pool, first/last 256 forced, budget 16384)
        pd = binding.pooled_desc(emb, qry, 16384, 129, 256, 256)
        wsp = torch.empty(binding.pooled_workspace_bytes(pd) + 256, dtype=torch.uint8, device=dev)
        psel = torch.empty((16384,), dtype=torch.int32, device=dev)
        ppool = torch.empty((N,), dtype=torch.float32, device=dev)
        pool_times = []
        for r in range(5):
            a, b = ev(), ev()
            a.record()
            binding.reform_gather_pooled(emb, qry, 16384, 129, 256, 256, sel_idx=psel, pooled=ppool,
                                         workspace=wsp)
            b.record()
            torch.cuda.synchronize()
            if r >= 2:
                pool_times.append(a.elapsed_time(b))
        # embedding construction for one chunk: 4 layers x 4 selected heads x C tokens, normalised into the store
        emb_times = []
        for r in range(5):
            a, b = ev(), ev()
            a.record()
            for layer in range(4):                    # one call per selected layer: its 4 heads
                binding.reform_embed_save_selected(out[4 * layer:4 * layer + 4], emb, 0, 4 * layer * d)
            b.record()
            torch.cuda.synchronize()
            if r >= 2:
                emb_times.append(a.elapsed_time(b))
        # the selected tokens' input embeddings (hidden 4096, bf16) gathered for recomputation
        table = torch.empty((N, 4096), dtype=torch.bfloat16, device=dev).normal_()
        rows_out = torch.empty((16384, 4096), dtype=torch.bfloat16, device=dev)
        rows_times = []
        for r in range(5):
            idx_r = ((psel.long() + r * 65537) % N).int()      # other rows every time: no cache reuse
            a, b = ev(), ev()
            a.record()
            binding.reform_gather_rows(table, idx_r, out=rows_out)
            b.record()
            torch.cuda.synchronize()
            if r >= 2:
                rows_times.append(a.elapsed_time(b))
        rows_times.sort()
        del table
        emb_times.sort()
        pool_times.sort()
        times.sort()
        sim_times.sort()
        g_ms = times[len(times) // 2]
        s_ms = sim_times[len(sim_times) // 2]
        g_bytes = float(N) * gcfg.D * 2 + 2.0 * gcfg.n_query * N * 4
        gather = {"workload": gcfg.name, "ms": g_ms, "min_ms": times[0],
                  "gbs": g_bytes / (g_ms * 1e-3) / 1e9, "frac_hbm": g_bytes / (g_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                  "similarity_ms": s_ms,
                  "similarity_gbs": (float(N) * gcfg.D * 2 + gcfg.n_query * N * 4.0) / (s_ms * 1e-3) / 1e9,
                  "union_count": int(uc.item()),
                  "pooled_ms": pool_times[len(pool_times) // 2],
                  "rows_ms": rows_times[len(rows_times) // 2],
                  "rows_gbs": 2.0 * 16384 * 8192 / (rows_times[len(rows_times) // 2] * 1e-3) / 1e9,
                  "embed_chunk_ms": emb_times[len(emb_times) // 2],
                  "embed_chunk_gbs": 16 * 2.0 * C * d * 2 / (emb_times[len(emb_times) // 2] * 1e-3) / 1e9,
                  "pooled_config": "max over 16 query tokens, window 129, forced 256+256, budget 16384"}

    line = {
        "metric": "context tokens/sec through chunk-compress at 1M ctx; gather top-k latency (ms)",
        "value": tok_s, "unit": "tokens/s", "n_gpus": 1, "steps": K_steps, "warmup": W_steps,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "zeros (debug)" if args.zero_data else "synthetic",
        "config": {"workload": cfg.name + " steady-state chunk (cache full), all layers",
                   "layers": layers, "q_heads": Hq, "kv_heads": Hkv, "head_dim": d, "chunk": C,
                   "budget": B, "obs_window": C, "gather": "cfg4_gather_1m: N=1048576 D=2048 nq=16 k=16384 r=8"},
        "gather_ms": None if gather is None else gather["ms"],
        "roofline": roof, "cpu_baseline": cpu, "kernels": kernels, "gather": gather,
        "paper_mode": paper_mode,
        "valid": layers == cfg.n_layers and not args.zero_data,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()

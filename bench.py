#!/usr/bin/env python3
"""Benchmark of the REFORM compress-and-gather hot path on one MI355X.

Headline: a step = one steady-state chunk of the 1M-token workload (C = B = 32768 tokens, cache
full) pushed through all 32 layers: per layer  reform_chunk_attend_score  (attention over
[cache || chunk] + eviction score) and  reform_evict_topk_compact  (top-B + compaction).  The
cache is first filled by an untimed chunk 0; inputs of every timed step are generated before the
timed region and sit in HBM.  value = context tokens/s through chunk-compress (steps * C / time).
After the timed steps the 1M-row gather (reform_gather_topk, 16 queries, k = 16384, radius 8) is
timed on its own and reported as gather_ms.

Beside the headline, in the same JSON line:
  full_pass        the whole 1M-token pass of that workload from an empty cache (32 chunks x 32
                   layers), L / sum of the time of the library calls
  configs          the other workloads (1, 2, 5: whole recurrence; 1, 2: their gather)
  measured_peaks   what this machine sustains in a pure bf16 MFMA loop, a plain copy and a
                   read-only stream (the library's probe kernels), so every fraction is given
                   against the data-sheet peak and against the measured ceiling
  cpu_baseline     the fp64 oracle on a bounded sample of the headline step, host cores stated;
                   cpu_baseline_configs: the oracle on whole workloads 1 and 4 (2 with a flag)
  paper_mode       the step as the paper's experiments configure the compressor

Prints ONE JSON line.
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
    ap.add_argument("--no-full-pass", action="store_true", help="skip the whole 1M-token pass (about 50 s)")
    ap.add_argument("--no-configs", action="store_true", help="skip the figures of workloads 1, 2 and 5")
    ap.add_argument("--oracle-configs", action="store_true",
                    help="also time the oracle on the whole of workload 2 (about ten minutes of CPU work)")
    ap.add_argument("--zero-data", action="store_true",
                    help="debug only: all-zero Q/K/V (marks the result invalid); shows how much of the "
                         "kernel time is the power-limited clock that random operands cause")
    ap.add_argument("--copy-probe", action="store_true",
                    help="after the timed region, run a plain 1 GiB -> 1 GiB elementwise copy kernel; "
                         "used to scale rocprofv3 FETCH_SIZE / WRITE_SIZE readings to bytes")
    return ap.parse_args()


def to_np(t):
    return t.detach().float().cpu().numpy()


def median(xs):
    xs = sorted(xs)
    return xs[len(xs) // 2]


def attn_flop(Hq, d, M, C):
    """Useful flop of one attention call: 4*d per unmasked (query, key) pair."""
    return 4.0 * d * Hq * (float(C) * M + C * (C + 1) / 2.0)


def evict_bytes(Hkv, n, B, d, elt):
    """Algorithmic bytes of one eviction: the candidate scores read, the retained K and V rows
    read and written (an upper bound: rows that keep their slot do not move)."""
    return Hkv * n * 4.0 + 2.0 * Hkv * min(n, B) * d * elt * 2


def cpu_baseline(cfg, q_mid, K, V, M):
    """The fp64 oracle, as it stands, on a bounded sample of the same layer-step: the middle
    rows of the chunk (their cost is the chunk's average), all heads, against the full
    [cache || chunk] key set, plus the per-head selection.  Extrapolated to 32 layers."""
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


def oracle_stream_pass(cfg, synth):
    """The oracle's own recurrence over a whole stream workload on the host (chunk attention +
    score, retention, compaction); returns seconds."""
    import numpy as np
    import oracle
    Hkv, d, cap = cfg.n_kv_heads, cfg.head_dim, cfg.capacity
    plan = synth.adversarial_plan(cfg) if cfg.kind == "adversarial" else None
    K = np.zeros((Hkv, cap, d), np.float32)
    V = np.zeros_like(K)
    M, dt = 0, 0.0
    for t in range(cfg.n_chunks):
        q, k, v = synth.chunk_qkv(cfg, 0, t, plan=plan)
        Ct = q.shape[1]
        K[:, M:M + Ct] = to_np(k)
        V[:, M:M + Ct] = to_np(v)
        qn = to_np(q)
        t0 = time.perf_counter()
        _, _, score = oracle.attend_score(qn, K, V, M, cfg.scale)
        K, V, _, _, _ = oracle.evict_compact(K, V, score, None, M + Ct, cfg.B)
        dt += time.perf_counter() - t0
        M = min(M + Ct, cfg.B)
        if dt > 20.0:                       # a long pass says where it is (stderr; stdout stays one JSON line)
            print(f"[bench] oracle pass of {cfg.name}: chunk {t + 1}/{cfg.n_chunks}, {dt:.0f} s", file=sys.stderr, flush=True)
    return dt


def gpu_store(raw, torch, binding, head_dim=128):
    """Embedding store of a "head_states" workload, built by the library's embedding-construction
    call from the raw head states [N, D] (untimed set-up of the gather figures)."""
    N, D = raw.shape
    store = torch.empty_like(raw)
    binding.reform_embed_save_selected(raw.view(N, D // head_dim, head_dim).permute(1, 0, 2), store, 0, 0)
    return store


def oracle_store(raw, torch, head_dim=128, block=65536):
    """The same store by the oracle's own routine from the same raw head states (host, float32
    view of the storage type), for the oracle's whole-workload gather time."""
    import numpy as np
    import oracle
    N, D = raw.shape
    out = np.empty((N, D), np.float32)
    for r0 in range(0, N, block):
        r1 = min(N, r0 + block)
        src = to_np(raw[r0:r1])
        emb = np.zeros((r1 - r0, D), np.float64)
        for h in range(D // head_dim):
            oracle.embed_segment(src[:, h * head_dim:(h + 1) * head_dim], emb, h * head_dim)
        out[r0:r1] = to_np(torch.from_numpy(emb).to(raw.dtype))
    return out


def measure_peaks(torch, binding, dev, big=None):
    """Pure bf16 MFMA loop (random operands), 1 GiB copy, read-only stream: best of five each."""
    ev = lambda: torch.cuda.Event(enable_timing=True)
    sink = torch.zeros((4,), dtype=torch.float32, device=dev)
    ops = torch.randn((32768,), device=dev).to(torch.bfloat16)            # 64 KiB of bf16
    best_mfma = 0.0
    for _ in range(6):
        a, b = ev(), ev()
        a.record()
        flop = binding.probe_mfma_bf16(ops, sink, 5000, 2048)
        b.record()
        torch.cuda.synchronize()
        best_mfma = max(best_mfma, flop / (a.elapsed_time(b) * 1e-3) / 1e12)
    src = torch.ones((1 << 28,), dtype=torch.int32, device=dev)           # 1 GiB
    dst = torch.empty_like(src)
    best_copy = 0.0
    for _ in range(6):
        a, b = ev(), ev()
        a.record()
        nbytes = binding.probe_stream(src, dst, sink)
        b.record()
        torch.cuda.synchronize()
        best_copy = max(best_copy, nbytes / (a.elapsed_time(b) * 1e-3) / 1e9)
    del dst
    rd = big if big is not None else src
    best_read = 0.0
    for _ in range(6):
        a, b = ev(), ev()
        a.record()
        nbytes = binding.probe_stream(rd, None, sink)
        b.record()
        torch.cuda.synchronize()
        best_read = max(best_read, nbytes / (a.elapsed_time(b) * 1e-3) / 1e9)
    return {"mfma_bf16_tflops": best_mfma, "hbm_copy_gbs": best_copy, "hbm_read_gbs": best_read,
            "how": "library probe kernels, best of 6: 16x16x32 bf16 MFMA loop on random operands "
                   "(2048 workgroups x 8 waves); 1 GiB -> 1 GiB copy (read + written bytes); read-only "
                   f"stream over {rd.numel() * rd.element_size() / 2**30:.1f} GiB"}


def run_stream_config(cfg, torch, binding, synth, dev):
    """Whole recurrence of a one-layer stream workload: every chunk through attend + score and
    evict + compact; the chunk's inputs are generated on the device outside the timed calls."""
    Hq, Hkv, d, C, B = cfg.n_q_heads, cfg.n_kv_heads, cfg.head_dim, cfg.C, cfg.B
    cap = cfg.capacity
    elt = 2 if cfg.dtype == torch.bfloat16 else 4
    plan = synth.adversarial_plan(cfg) if cfg.kind == "adversarial" else None
    K = torch.zeros((Hkv, cap, d), dtype=cfg.dtype, device=dev)
    V = torch.zeros_like(K)
    score = torch.zeros((Hkv, cap), dtype=torch.float32, device=dev)
    pos = torch.zeros((Hkv, cap), dtype=torch.int32, device=dev)
    out = torch.empty((Hq, C, d), dtype=cfg.dtype, device=dev)
    lse = torch.empty((Hq, C), dtype=torch.float32, device=dev)
    kept = torch.empty((Hkv, B), dtype=torch.int32, device=dev)
    ws_e = torch.empty(binding.evict_workspace_bytes(binding.evict_desc(K, min(B + C, cap), B)) + 256,
                       dtype=torch.uint8, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks, M = [], 0
    for t in range(cfg.n_chunks):
        q, k, v = synth.chunk_qkv(cfg, 0, t, dev, plan=plan)
        Ct = q.shape[1]
        K[:, M:M + Ct] = k
        V[:, M:M + Ct] = v
        pos[:, M:M + Ct] = torch.arange(t * C, t * C + Ct, dtype=torch.int32, device=dev)
        e = [ev(), ev(), ev()]
        e[0].record()
        binding.reform_chunk_attend_score(q, K, V, M, cfg.scale, out=out[:, :Ct],
                                          lse=lse.view(-1)[:Hq * Ct].view(Hq, Ct), score=score)
        e[1].record()
        binding.reform_evict_topk_compact(K, V, score, M + Ct, B, pos=pos, kept_idx=kept, workspace=ws_e)
        e[2].record()
        marks.append((e, M, Ct))
        M = min(M + Ct, B)
    torch.cuda.synchronize()
    att = [e[0].elapsed_time(e[1]) for e, _, _ in marks]
    evi = [e[1].elapsed_time(e[2]) for e, _, _ in marks]
    total_ms = sum(att) + sum(evi)
    flop = sum(attn_flop(Hq, d, M_, Ct) for _, M_, Ct in marks)
    steady = [i for i, (_, M_, Ct) in enumerate(marks) if M_ == B and Ct == C]
    res = {"workload": cfg.name, "dtype": "bf16" if elt == 2 else "f32", "chunks": cfg.n_chunks,
           "tokens_per_s": cfg.L / (total_ms * 1e-3), "pass_ms": total_ms,
           "attend_ms_total": sum(att), "evict_ms_total": sum(evi),
           "attend_tflops_useful": flop / (sum(att) * 1e-3) / 1e12}
    if elt == 2:
        res["attend_frac_mfma_useful"] = res["attend_tflops_useful"] / PEAK_BF16_TFLOPS
    if steady:
        a_ms = median([att[i] for i in steady])
        e_ms = median([evi[i] for i in steady])
        eb = evict_bytes(Hkv, B + C, B, d, elt)
        res.update(steady_attend_ms=a_ms, steady_evict_ms=e_ms,
                   steady_evict_gbs=eb / (e_ms * 1e-3) / 1e9,
                   steady_evict_frac_hbm=eb / (e_ms * 1e-3) / 1e9 / PEAK_HBM_GBS)
    return res


def run_gather_config(gcfg, torch, binding, synth, dev, sets):
    """Median of five reform_gather_topk calls; `sets` distinct copies of the inputs are used in
    turn so that a store smaller than the last-level cache is read from HBM every time."""
    data = [synth.gather_inputs(synth.scaled(gcfg, seed=gcfg.seed + 1000 * s), dev) for s in range(sets)]
    N = gcfg.N
    elt = 2 if gcfg.dtype == torch.bfloat16 else 4
    gd = binding.gather_desc(data[0][0], data[0][1], gcfg.k, gcfg.radius)
    ws = torch.empty(binding.gather_workspace_bytes(gd) + 256, dtype=torch.uint8, device=dev)
    ti = torch.empty((gcfg.n_query, gcfg.k), dtype=torch.int32, device=dev)
    ts = torch.empty((gcfg.n_query, gcfg.k), dtype=torch.float32, device=dev)
    ui = torch.empty((N,), dtype=torch.int32, device=dev)
    uc = torch.zeros((1,), dtype=torch.int32, device=dev)
    ev = lambda: torch.cuda.Event(enable_timing=True)
    times = []
    for r in range(3 + 5):
        emb, qry = data[r % sets]
        a, b = ev(), ev()
        a.record()
        binding.reform_gather_topk(emb, qry, gcfg.k, gcfg.radius, topk_idx=ti, topk_score=ts,
                                   union_idx=ui, union_count=uc, workspace=ws)
        b.record()
        torch.cuda.synchronize()
        if r >= 3:
            times.append(a.elapsed_time(b))
    ms = median(times)
    nbytes = float(N) * gcfg.D * elt + 2.0 * gcfg.n_query * N * 4
    return {"workload": gcfg.name, "ms": ms, "min_ms": min(times), "gbs": nbytes / (ms * 1e-3) / 1e9,
            "frac_hbm": nbytes / (ms * 1e-3) / 1e9 / PEAK_HBM_GBS, "input_sets_rotated": sets}


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

    def fill_chunk0():
        tok0 = torch.arange(C, dtype=torch.int32, device=dev)
        for l, (q, k, v) in enumerate(gen(0)):
            Kc[l][:, :C] = k
            Vc[l][:, :C] = v
            pos[l][:, :C] = tok0
            binding.reform_chunk_attend_score(q, Kc[l], Vc[l], 0, cfg.scale, out=out, lse=lse, score=score,
                                              workspace=ws_attn)
            binding.reform_evict_topk_compact(Kc[l], Vc[l], score, C, B, pos=pos[l], kept_idx=kept,
                                              workspace=ws_evict)

    # ---- untimed fill: chunk 0 with an empty cache
    fill_chunk0()
    M = min(C, B)
    torch.cuda.synchronize()
    inputs = [gen(1 + s) for s in range(pool)]
    torch.cuda.synchronize()

    ev = lambda: torch.cuda.Event(enable_timing=True)
    marks = []                                 # (e0, e1, e2, e3) per timed layer-step

    mode = {"obs_window": 0, "n_sink": 0, "n_recent": 0, "rope": False}   # default workload: W = C, nothing forced

    def layer_step(l, q, k, v, M_, tok, timed):
        """One layer of one chunk: the chunk's K/V land at rows [M, M+C) (in a model: written there
        by the QKV projection; per head the copy is contiguous), then the two library calls."""
        W, ns, nr = mode["obs_window"], mode["n_sink"], mode["n_recent"]
        Ct = q.shape[1]
        for h in range(Hkv):
            Kc[l][h, M_:M_ + Ct].copy_(k[h])
            Vc[l][h, M_:M_ + Ct].copy_(v[h])
        pos[l][:, M_:M_ + Ct] = tok
        if timed:
            e = [ev() for _ in range(5)]
            e[0].record()
            binding.reform_chunk_attend_score(q, Kc[l], Vc[l], M_, cfg.scale, obs_window=W, out=out,
                                              lse=lse, score=score, workspace=ws_attn, phases=1)
            e[1].record()
            binding.reform_chunk_attend_score(q, Kc[l], Vc[l], M_, cfg.scale, obs_window=W, out=out,
                                              lse=lse, score=score, workspace=ws_attn, phases=2)
            e[2].record()
            binding.reform_evict_topk_compact(Kc[l], Vc[l], score, M_ + Ct, B, ns, nr, pos=pos[l],
                                              kept_idx=kept, workspace=ws_evict)
            e[3].record()
            if mode["rope"]:
                binding.reform_rerotate_keys(Kc[l], kept, B, 1e6)
            e[4].record()
            marks.append(e)
        else:
            binding.reform_chunk_attend_score(q, Kc[l], Vc[l], M_, cfg.scale, obs_window=W, out=out,
                                              lse=lse, score=score, workspace=ws_attn)
            binding.reform_evict_topk_compact(Kc[l], Vc[l], score, M_ + Ct, B, ns, nr, pos=pos[l],
                                              kept_idx=kept, workspace=ws_evict)
            if mode["rope"]:
                binding.reform_rerotate_keys(Kc[l], kept, B, 1e6)

    def step(s, timed):
        data = inputs[s % pool]
        tok = torch.arange((1 + s) * C, (2 + s) * C, dtype=torch.int32, device=dev)
        for l in range(layers):
            q, k, v = data[l]
            layer_step(l, q, k, v, M, tok, timed)

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

    fwd_flop = attn_flop(Hq, d, M, C)          # QK^T + PV on unmasked pairs
    sc_flop = fwd_flop / 2.0                   # second QK^T of the exact score (executed, not useful)
    ev_bytes = evict_bytes(Hkv, M + C, B, d, 2)
    roof = {"kernel": "attn_fwd_bf16", "bound": "mfma", "achieved": fwd_flop / (fwd_ms * 1e-3) / 1e12,
            "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "traffic": FWD_TRAFFIC_BYTES,
            "traffic_source": "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, profiles/attn_fwd_cfg3_hbm_traffic.md"}
    roof["frac"] = roof["achieved"] / roof["peak"]
    kernels = {
        "attn_fwd_bf16": {"ms": fwd_ms, "tflops": roof["achieved"], "frac_mfma": roof["frac"]},
        "attn_score_bf16": {"ms": sc_ms, "tflops_executed": sc_flop / (sc_ms * 1e-3) / 1e12,
                            "frac_mfma": sc_flop / (sc_ms * 1e-3) / 1e12 / PEAK_BF16_TFLOPS},
        "attend_call": {"ms": fwd_ms + sc_ms,
                        "tflops_useful": fwd_flop / ((fwd_ms + sc_ms) * 1e-3) / 1e12,
                        "tflops_executed": (fwd_flop + sc_flop) / ((fwd_ms + sc_ms) * 1e-3) / 1e12},
        "evict_call": {"ms": evict_ms, "gbs": ev_bytes / (evict_ms * 1e-3) / 1e9,
                       "frac_hbm": ev_bytes / (evict_ms * 1e-3) / 1e9 / PEAK_HBM_GBS},
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
    mode.update(obs_window=0, n_sink=0, n_recent=0, rope=False)

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
        q, k, v = inputs[0][0]
        half = 512
        rows = slice(C // 2 - half, C // 2 + half)
        Mo = M + C // 2 - half
        Kh = torch.cat([Kc[0][:, :M], k[:, :C // 2 + half]], dim=1)
        Vh = torch.cat([Vc[0][:, :M], v[:, :C // 2 + half]], dim=1)
        cpu = cpu_baseline(cfg, to_np(q[:, rows]), to_np(Kh), to_np(Vh), Mo)
        del Kh, Vh
    del inputs
    torch.cuda.empty_cache()

    # ---- the whole 1M-token pass from an empty cache: 32 chunks, every layer; only the library
    # calls and the chunk's K/V placement are inside the summed time, generation is not
    full_pass = None
    if not args.no_full_pass:
        Mf, sec, chunk_ms = 0, 0.0, []
        for t in range(cfg.n_chunks):
            data = gen(t)
            tok = torch.arange(t * C, (t + 1) * C, dtype=torch.int32, device=dev)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            for l in range(layers):
                q, k, v = data[l]
                layer_step(l, q, k, v, Mf, tok, False)
            torch.cuda.synchronize()
            dt = time.perf_counter() - t2
            sec += dt
            chunk_ms.append(dt * 1e3)
            Mf = min(Mf + C, B)
            del data
        full_pass = {"workload": cfg.name + ", every chunk from an empty cache", "chunks": cfg.n_chunks,
                     "layers": layers, "tokens": cfg.L, "seconds": sec, "tokens_per_s": cfg.L / sec,
                     "first_chunk_ms": chunk_ms[0], "steady_chunk_ms": median(chunk_ms[1:]),
                     "useful_pflop": sum(attn_flop(Hq, d, min(t * C, B), C) for t in range(cfg.n_chunks)) * layers / 1e15}
        full_pass["useful_tflops"] = full_pass["useful_pflop"] * 1e3 / sec
    del Kc, Vc, pos
    torch.cuda.empty_cache()

    # ---- the other stream workloads and their gathers
    configs = None
    if not args.no_configs:
        configs = {}
        for cid in (1, 2, 5):
            configs[str(cid)] = {"stream": run_stream_config(synth.STREAMS[cid], torch, binding, synth, dev)}
        configs["1"]["gather"] = run_gather_config(synth.GATHERS[1], torch, binding, synth, dev, sets=4)
        configs["2"]["gather"] = run_gather_config(synth.GATHERS[2], torch, binding, synth, dev, sets=3)
        torch.cuda.empty_cache()

    # ---- gather at 1M rows
    gather, peaks, cpu_cfgs = None, None, None
    emb = None
    if not args.no_gather:
        gcfg = synth.GATHERS[4]
        emb_raw, qry_raw = synth.gather_inputs(gcfg, dev)       # raw head states
        emb, qry = gpu_store(emb_raw, torch, binding), gpu_store(qry_raw, torch, binding)
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
        # embedding construction for one chunk: 4 layers x 4 selected heads x C tokens, normalised
        # into a store of the same shape (a scratch copy: the timed store above stays untouched)
        emb_times = []
        store = torch.empty((C, gcfg.D), dtype=torch.bfloat16, device=dev)
        for r in range(5):
            a, b = ev(), ev()
            a.record()
            for layer in range(4):                    # one call per selected layer: its 4 heads
                binding.reform_embed_save_selected(out[4 * layer:4 * layer + 4], store, 0, 4 * layer * d)
            b.record()
            torch.cuda.synchronize()
            if r >= 2:
                emb_times.append(a.elapsed_time(b))
        del store
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
        del table
        g_ms = median(times)
        s_ms = median(sim_times)
        g_bytes = float(N) * gcfg.D * 2 + 2.0 * gcfg.n_query * N * 4
        gather = {"workload": gcfg.name, "ms": g_ms, "min_ms": min(times),
                  "gbs": g_bytes / (g_ms * 1e-3) / 1e9, "frac_hbm": g_bytes / (g_ms * 1e-3) / 1e9 / PEAK_HBM_GBS,
                  "similarity_ms": s_ms,
                  "similarity_gbs": (float(N) * gcfg.D * 2 + gcfg.n_query * N * 4.0) / (s_ms * 1e-3) / 1e9,
                  "union_count": int(uc.item()),
                  "pooled_ms": median(pool_times),
                  "rows_ms": median(rows_times),
                  "rows_gbs": 2.0 * 16384 * 8192 / (median(rows_times) * 1e-3) / 1e9,
                  "embed_chunk_ms": median(emb_times),
                  "embed_chunk_gbs": 16 * 2.0 * C * d * 2 / (median(emb_times) * 1e-3) / 1e9,
                  "pooled_config": "max over 16 query tokens, window 129, forced 256+256, budget 16384"}

    # ---- measured ceilings of this machine, and every fraction against them as well
    peaks = measure_peaks(torch, binding, dev, big=emb)
    roof["peak_measured"] = peaks["mfma_bf16_tflops"]
    roof["frac_measured"] = roof["achieved"] / peaks["mfma_bf16_tflops"]
    kernels["attn_score_bf16"]["frac_mfma_measured"] = kernels["attn_score_bf16"]["tflops_executed"] / peaks["mfma_bf16_tflops"]
    kernels["evict_call"]["peak_measured_gbs"] = peaks["hbm_copy_gbs"]
    kernels["evict_call"]["frac_measured"] = kernels["evict_call"]["gbs"] / peaks["hbm_copy_gbs"]
    if gather is not None:
        gather["peak_measured_gbs"] = peaks["hbm_read_gbs"]
        gather["frac_measured"] = gather["gbs"] / peaks["hbm_read_gbs"]

    # ---- the oracle on whole workloads (host cores), after every GPU figure is taken
    if not args.no_cpu_baseline:
        import oracle
        cpu_cfgs = {"cores": oracle.num_threads(), "kind": "oracle, whole workload"}
        c1 = synth.STREAMS[1]
        s1 = oracle_stream_pass(c1, synth)
        e1, q1 = synth.gather_inputs(synth.GATHERS[1])
        t3 = time.perf_counter()
        oracle.gather(to_np(e1), to_np(q1), synth.GATHERS[1].k, synth.GATHERS[1].radius)
        g1 = time.perf_counter() - t3
        cpu_cfgs["1"] = {"stream_seconds": s1, "stream_tokens_per_s": c1.L / s1, "gather_ms": g1 * 1e3}
        if emb is not None:
            gcfg = synth.GATHERS[4]
            del emb
            en, qn = oracle_store(emb_raw, torch), oracle_store(qry_raw, torch)
            t3 = time.perf_counter()
            oracle.gather(en, qn, gcfg.k, gcfg.radius)
            cpu_cfgs["4"] = {"gather_ms": (time.perf_counter() - t3) * 1e3}
            del en, qn
        if args.oracle_configs:
            c2 = synth.STREAMS[2]
            s2 = oracle_stream_pass(c2, synth)
            e2, q2 = synth.gather_inputs(synth.GATHERS[2])
            t3 = time.perf_counter()
            oracle.gather(to_np(e2), to_np(q2), synth.GATHERS[2].k, synth.GATHERS[2].radius)
            cpu_cfgs["2"] = {"stream_seconds": s2, "stream_tokens_per_s": c2.L / s2,
                             "gather_ms": (time.perf_counter() - t3) * 1e3,
                             "stream_threads": min(oracle.num_threads(), c2.n_kv_heads)}

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
        "full_pass": full_pass, "configs": configs, "measured_peaks": peaks,
        "cpu_baseline_configs": cpu_cfgs, "paper_mode": paper_mode,
        "valid": layers == cfg.n_layers and not args.zero_data,
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()

"""GPU parity: reform_evict_topk_compact against the CPU oracle, bit-exact.

The call takes fp32 scores as input, so both sides decide on identical numbers and every
output (kept indices, K, V, score, pos rows) must match exactly, ties included."""
import numpy as np
import pytest
import torch

import oracle
from helpers import to_np
from paper_2506_01215_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_case(Hkv, d, n, B, cap, dtype, score, n_sink=0, n_recent=0, seed=0, with_pos=True, with_kept=True):
    print(f"[evict] Hkv={Hkv} d={d} n={n} B={B} cap={cap} {dtype} sink={n_sink} recent={n_recent}", flush=True)
    g = torch.Generator().manual_seed(seed)
    k = torch.randn((Hkv, cap, d), generator=g).to(dtype)
    v = torch.randn((Hkv, cap, d), generator=g).to(dtype)
    pos = (torch.arange(cap, dtype=torch.int32) * 3 + 7).repeat(Hkv, 1).contiguous()
    kd, vd, sd = k.to(DEV), v.to(DEV), score.to(DEV)
    pd = pos.to(DEV) if with_pos else None
    kept = torch.full((Hkv, B), -1, dtype=torch.int32, device=DEV) if with_kept else None
    ws = torch.full((binding.evict_workspace_bytes(binding.evict_desc(kd, n, B, n_sink, n_recent)) + 256,), 0x5a,
                    dtype=torch.uint8, device=DEV)
    new_len = binding.reform_evict_topk_compact(kd, vd, sd, n, B, n_sink, n_recent, pos=pd, kept_idx=kept,
                                                workspace=ws)
    torch.cuda.synchronize()
    assert new_len == min(n, B)
    if n > B and 16384 % (d * k.element_size()) == 0:
        # in-place move: the device-side status word (first int32 of the aligned workspace) stays 0
        assert binding.evict_status_word(ws) == 0
    k2, v2, s2, p2, kept_ref = oracle.evict_compact(to_np(k), to_np(v), to_np(score).astype(np.float64),
                                                    pos.numpy(), n, B, n_sink, n_recent)
    if with_kept:
        np.testing.assert_array_equal(kept.cpu().numpy()[:, :new_len], kept_ref)
        assert (kept.cpu().numpy()[:, new_len:] == -1).all()
    np.testing.assert_array_equal(to_np(kd)[:, :new_len], k2[:, :new_len])
    np.testing.assert_array_equal(to_np(vd)[:, :new_len], v2[:, :new_len])
    np.testing.assert_array_equal(sd.cpu().numpy()[:, :new_len].astype(np.float64), s2[:, :new_len])
    if with_pos:
        np.testing.assert_array_equal(pd.cpu().numpy()[:, :new_len], p2[:, :new_len])
    # rows past the candidates are never touched
    np.testing.assert_array_equal(to_np(kd)[:, n:], to_np(k)[:, n:])
    np.testing.assert_array_equal(to_np(vd)[:, n:], to_np(v)[:, n:])
    return kept_ref


def rand_scores(Hkv, cap, seed, ties=False):
    g = torch.Generator().manual_seed(seed)
    if ties:
        return torch.randint(0, 7, (Hkv, cap), generator=g).float() * 0.25
    return torch.rand((Hkv, cap), generator=g) * 3.0


@pytest.mark.parametrize("Hkv,d,n,B,dtype,ties", [
    (4, 64, 384, 256, torch.float32, False),      # workload 1
    (2, 128, 1000, 333, torch.bfloat16, False),
    (3, 128, 5000, 4096, torch.bfloat16, True),   # heavy ties
    (8, 128, 4113, 4096, torch.bfloat16, True),   # workload 5's ragged tail: 17 evictions
    (2, 64, 20000, 1, torch.bfloat16, False),     # budget of one
    (1, 128, 9000, 8999, torch.float32, True),    # evict exactly one
    (8, 128, 20480, 4096, torch.bfloat16, True),  # workload 5 steady state
])
def test_matches_oracle(Hkv, d, n, B, dtype, ties):
    cap = n + 9
    run_case(Hkv, d, n, B, cap, dtype, rand_scores(Hkv, cap, n + B, ties), seed=n)


@pytest.mark.parametrize("Hkv,n,B,pad,ties,sink,recent", [
    (2, 4096, 2000, 0, True, 0, 0),         # one step per lane, aligned rows
    (2, 4097, 4000, 3, True, 5, 9),         # first size of the four-step variant, unaligned pitch
    (2, 16384, 8000, 0, False, 0, 0),
    (1, 16385, 100, 2, True, 0, 3),         # first size of the sixteen-step variant
    (2, 65535, 32768, 1, True, 0, 0),       # ragged last quad at the largest single-launch size
    (1, 65536, 65535, 0, True, 0, 0),       # evict exactly one of 65536
    (2, 65536, 30000, 0, True, 256, 256),
    (2, 65537, 30000, 3, True, 0, 0),       # first size of the multi-launch selection
    (2, 70001, 30000, 3, True, 256, 256),
    (1, 131072, 1000, 0, False, 0, 0),
    (8, 65536, 32768, 0, True, 0, 0),       # 16 workgroups per row in the one-launch selection of long rows
    (3, 300000, 123456, 1, True, 7, 9),     # several candidates blocks per workgroup there, ragged
    (33, 140001, 50000, 3, True, 0, 0),     # too many workgroups for one launch: the multi-launch selection
    (1, 600001, 250000, 1, True, 2, 2),     # 8192 keys per workgroup of the one-launch selection
    (1, 3000000, 1000, 0, False, 0, 0),     # 32768 keys per workgroup, 92 workgroups for the one row
])
def test_selection_paths(Hkv, n, B, pad, ties, sink, recent):
    """Sizes on both sides of every switch inside the selection (registers per lane, one workgroup
    per row, several workgroups per row in one launch, several launches), with ties, forced slots
    and rows that cannot be read as aligned quads."""
    cap = n + pad
    run_case(Hkv, 64, n, B, cap, torch.bfloat16, rand_scores(Hkv, cap, n + B + pad, ties), sink, recent, seed=n)


def test_constant_and_two_valued_scores_at_full_size():
    """Every candidate in one histogram bin (the whole-wave shortcut of the single-launch selection)."""
    kept = run_case(2, 64, 65536, 32768, 65536, torch.bfloat16, torch.full((2, 65536), 0.37))
    assert (kept == np.arange(32768)).all()
    s = torch.full((2, 65536), 1.0)
    s[:, 40000:] = 1.0000001
    kept = run_case(2, 64, 65536, 32768, 65536, torch.bfloat16, s)
    assert (kept[:, :7232] == np.arange(7232)).all() and (kept[:, 7232:] == np.arange(40000, 65536)).all()


def test_all_scores_equal_keeps_the_first_B():
    kept = run_case(2, 64, 3000, 1200, 3000, torch.bfloat16, torch.ones((2, 3000)))
    assert (kept == np.arange(1200)).all()


def test_negative_zero_and_signed_scores():
    s = rand_scores(2, 700, 3) - 1.5
    s[:, ::5] = 0.0
    s[:, 1::5] = -0.0
    run_case(2, 64, 700, 300, 700, torch.float32, s)


def test_sinks_and_recents_are_protected():
    s = rand_scores(4, 2100, 5, ties=True)
    s[:, :8] = -1.0
    s[:, 2000 - 16:2000] = -1.0
    run_case(4, 128, 2000, 512, 2100, torch.bfloat16, s, n_sink=8, n_recent=16)
    run_case(4, 128, 2000, 512, 2100, torch.bfloat16, s, n_sink=256, n_recent=256)
    run_case(4, 128, 2000, 512, 2100, torch.bfloat16, s, n_sink=0, n_recent=512)


@pytest.mark.parametrize("pattern", ["keep_last", "keep_every_other", "keep_first", "keep_blocks"])
def test_in_place_hazard_patterns(pattern):
    """Keep sets that maximise the overlap between source and destination rows."""
    Hkv, n, B = 2, 8192, 4096
    j = torch.arange(n).float()
    if pattern == "keep_last":
        s = j.clone()
    elif pattern == "keep_every_other":
        s = (torch.arange(n) % 2).float()
        s[1::2] += 1.0
    elif pattern == "keep_first":
        s = -j
    else:
        s = ((torch.arange(n) // 37) % 2).float() + 0.001 * torch.rand(n, generator=torch.Generator().manual_seed(1))
    s = s.repeat(Hkv, 1).contiguous()
    run_case(Hkv, 128, n, B, n, torch.bfloat16, s)


def test_nothing_to_evict_moves_nothing():
    Hkv, d, n, B, cap = 2, 128, 300, 512, 600
    g = torch.Generator().manual_seed(9)
    k = torch.randn((Hkv, cap, d), generator=g).bfloat16().to(DEV)
    v = torch.randn((Hkv, cap, d), generator=g).bfloat16().to(DEV)
    s = torch.rand((Hkv, cap), generator=g).to(DEV)
    k0, v0, s0 = k.clone(), v.clone(), s.clone()
    kept = torch.full((Hkv, B), -1, dtype=torch.int32, device=DEV)
    assert binding.reform_evict_topk_compact(k, v, s, n, B, kept_idx=kept) == n
    torch.cuda.synchronize()
    assert torch.equal(k, k0) and torch.equal(v, v0) and torch.equal(s, s0)
    assert (kept[:, :n].cpu() == torch.arange(n, dtype=torch.int32)).all() and (kept[:, n:] == -1).all()


def test_optional_outputs_may_be_null():
    run_case(2, 64, 900, 400, 900, torch.bfloat16, rand_scores(2, 900, 2), with_pos=False, with_kept=False)


def test_row_size_that_needs_the_staged_path():
    """head_dim 96 bf16 = 192-byte rows: not a divisor of the 16 KB in-place tile."""
    run_case(3, 96, 3000, 1000, 3010, torch.bfloat16, rand_scores(3, 3010, 8, ties=True), seed=4)
    run_case(2, 24, 500, 200, 500, torch.float32, rand_scores(2, 500, 9), seed=5)


def test_full_size_layer_step():
    """Workload 3's shape: 8 KV heads, 65536 candidates -> 32768, head_dim 128 bf16."""
    run_case(8, 128, 65536, 32768, 65536, torch.bfloat16, rand_scores(8, 65536, 77, ties=False), seed=3)


def test_bounded_wait_gives_up_and_reports():
    """The in-place move's give-up branch, forced from the host: with a poll limit of 0 no tile
    publishes and every wait on another tile expires at once, so the call still ends (every kernel
    runs to completion) and the status word says that the cache is not to be trusted.  With the
    default limit restored the same problem is exact again and the word stays 0."""
    Hkv, n, B, d = 2, 8192, 4096, 128
    s = (torch.arange(n) % 2).float().repeat(Hkv, 1).contiguous()     # keeps every other row: tiles depend on earlier tiles
    g = torch.Generator().manual_seed(11)
    k = torch.randn((Hkv, n, d), generator=g).bfloat16().to(DEV)
    v = torch.randn((Hkv, n, d), generator=g).bfloat16().to(DEV)
    ws = torch.zeros((binding.evict_workspace_bytes(binding.evict_desc(k, n, B)) + 256,), dtype=torch.uint8, device=DEV)
    print("[evict] forced give-up of the bounded wait", flush=True)
    binding.debug_set_move_spin_limit(0)
    try:
        binding.reform_evict_topk_compact(k, v, s.to(DEV), n, B, workspace=ws)
        torch.cuda.synchronize()
        assert binding.evict_status_word(ws) == 1
    finally:
        binding.debug_set_move_spin_limit(-1)
    run_case(Hkv, d, n, B, n, torch.bfloat16, s)                        # asserts exact results and a clear status word

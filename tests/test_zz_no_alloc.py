"""GPU: reform_evict_topk_compact_static (the entry point for callers that cannot allocate: its
scratch is a static device array inside the library) against reform_evict_topk_compact with a
caller workspace.  Integer and byte work, so every output must be bit-identical.  Two calls in a
row share the static array; the second is smaller, so it runs over the first call's leftovers."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2506_01215_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def make_case(Hkv, d, n, B, cap, seed, ties):
    g = torch.Generator().manual_seed(seed)
    k = torch.randn((Hkv, cap, d), generator=g).bfloat16()
    v = torch.randn((Hkv, cap, d), generator=g).bfloat16()
    if ties:
        s = torch.randint(0, 9, (Hkv, cap), generator=g).float() * 0.125
    else:
        s = torch.rand((Hkv, cap), generator=g) * 3.0
    pos = (torch.arange(cap, dtype=torch.int32) * 5 + 11).repeat(Hkv, 1).contiguous()
    return k, v, s, pos


def run_both(Hkv, d, n, B, cap, seed, ties, n_sink=0, n_recent=0):
    print(f"[no-alloc evict] Hkv={Hkv} d={d} n={n} B={B} cap={cap} seed={seed} ties={ties}", flush=True)
    k, v, s, pos = make_case(Hkv, d, n, B, cap, seed, ties)
    ref = [t.to(DEV) for t in (k, v, s, pos)]
    got = [t.to(DEV) for t in (k, v, s, pos)]
    kept_ref = torch.full((Hkv, B), -1, dtype=torch.int32, device=DEV)
    kept_got = torch.full((Hkv, B), -1, dtype=torch.int32, device=DEV)
    new_len = binding.reform_evict_topk_compact(ref[0], ref[1], ref[2], n, B, n_sink, n_recent,
                                                pos=ref[3], kept_idx=kept_ref)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    assert binding.reform_evict_topk_compact_static(got[0], got[1], got[2], n, B, n_sink, n_recent,
                                                    pos=got[3], kept_idx=kept_got) == new_len
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before          # the binding allocated nothing either
    assert torch.equal(kept_got, kept_ref)
    for a, b, name in zip(got, ref, ("k", "v", "score", "pos")):
        assert torch.equal(a[:, :new_len], b[:, :new_len]), name
        assert torch.equal(a[:, n:], b[:, n:]), name + " beyond the candidates"
    return kept_got


def test_two_calls_in_a_row_second_smaller():
    # workload 3's layer-step shape (multi-launch selection, in-place move, 5.3 MB of scratch) ...
    run_both(8, 128, 65536, 32768, 65536, seed=1, ties=False)
    # ... then a smaller, ragged, tie-heavy one (single-launch selection) over the same scratch
    run_both(8, 128, 20480, 4096, 20489, seed=2, ties=True, n_sink=4, n_recent=16)
    # ... a staged (not in-place) row size and a call with nothing to evict
    run_both(3, 96, 3000, 1000, 3010, seed=3, ties=True)
    run_both(2, 128, 300, 512, 600, seed=4, ties=False)
    # and the large one again after the small ones
    run_both(8, 128, 65536, 32768, 65536, seed=5, ties=True)


def test_rejects_what_does_not_fit_the_static_scratch():
    lib = binding.load_library()
    Hkv, d, n, B = 64, 128, 131072, 65536                    # needs far more than 8 MiB
    desc = binding.EvictDesc(ctypes.sizeof(binding.EvictDesc), binding.REFORM_BF16, Hkv, d, n, B, n, 0, 0)
    assert lib.reform_evict_topk_compact_workspace(ctypes.byref(desc)) > binding.STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)
    rc = lib.reform_evict_topk_compact_static(ctypes.byref(desc), fake, fake, fake, None, None, None)
    assert rc == 3                                           # REFORM_ERR_WORKSPACE, nothing launched

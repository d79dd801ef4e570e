"""GPU parity of reform_rerotate_keys (consecutive position ids after compression, Sec. 3.1)
against the fp64 oracle, on caches compacted by reform_evict_topk_compact."""
import numpy as np
import pytest
import torch

import oracle
from helpers import RTOL, assert_close, to_np
from paper_2506_01215_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def run_case(Hkv, d, n, B, dtype, theta, rot, seed):
    g = torch.Generator().manual_seed(seed)
    cap = n + 5
    k = torch.randn((Hkv, cap, d), generator=g).to(dtype)
    v = torch.randn((Hkv, cap, d), generator=g).to(dtype)
    score = torch.rand((Hkv, cap), generator=g)
    kd, vd, sd = k.to(DEV), v.to(DEV), score.to(DEV)
    kept = torch.full((Hkv, B), -1, dtype=torch.int32, device=DEV)
    print(f"[rope] Hkv={Hkv} d={d} n={n} B={B} dtype={dtype} theta={theta} rot={rot}", flush=True)
    new_len = binding.reform_evict_topk_compact(kd, vd, sd, n, B, n_sink=3, kept_idx=kept)
    compact, v_after_evict = kd.clone(), vd.clone()
    binding.reform_rerotate_keys(kd, kept, new_len, theta, rot)
    torch.cuda.synchronize()
    kept_h = kept.cpu().numpy()
    got, before = to_np(kd), to_np(compact)
    for h in range(Hkv):
        want = oracle.rerotate_keys(before[h, :new_len], kept_h[h, :new_len], theta, rot)
        assert_close(got[h, :new_len], want, RTOL[dtype], f"head {h}")
        same = kept_h[h, :new_len] == np.arange(new_len)
        assert same[:3].all()                                            # the sinks never move
        np.testing.assert_array_equal(got[h, :new_len][same], before[h, :new_len][same])
        nrm_b = np.linalg.norm(before[h, :new_len].astype(np.float64), axis=1)
        nrm_a = np.linalg.norm(got[h, :new_len].astype(np.float64), axis=1)
        np.testing.assert_allclose(nrm_a, nrm_b, rtol=4e-3 if dtype == torch.bfloat16 else 1e-6)
    np.testing.assert_array_equal(got[:, new_len:], before[:, new_len:])  # rows past the cache untouched
    assert torch.equal(vd, v_after_evict)                                  # V carries no rotary embedding
    return got


@pytest.mark.parametrize("Hkv,d,n,B,dtype,theta,rot", [
    (4, 64, 384, 256, torch.float32, 10000.0, None),        # workload 1 shape
    (2, 128, 3000, 1000, torch.bfloat16, 1e6, None),        # the evaluated models' base and head_dim
    (8, 128, 20480, 4096, torch.bfloat16, 10000.0, None),   # workload 5 steady state: deltas up to -16384
    (2, 128, 700, 300, torch.bfloat16, 10000.0, 64),        # partial rotary dimension
    (1, 32, 500, 100, torch.float32, 500.0, 16),
    (2, 64, 100, 200, torch.bfloat16, 10000.0, None),       # n <= B: nothing moved, nothing rotated
    (2, 128, 300, 100, torch.bfloat16, 10000.0, 0),         # rotary_dim 0: a no-op
])
def test_matches_oracle(Hkv, d, n, B, dtype, theta, rot):
    run_case(Hkv, d, n, B, dtype, theta, rot, seed=n + B)


def test_full_size_layer_step():
    """8 heads x 65536 candidates -> 32768 retained rows of 128 bf16: the shape bench.py times."""
    run_case(8, 128, 65536, 32768, torch.bfloat16, 1e6, None, seed=1)

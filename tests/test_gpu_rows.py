"""GPU parity of reform_gather_rows (the inputs gathered for recomputation, Sec. 3.3 / Alg. 1):
byte-exact against the oracle, including the device-side count and the bad-index flag."""
import numpy as np
import pytest
import torch

import oracle
from paper_2506_01215_amd import binding

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def raw(t):
    return t.cpu().contiguous().view(torch.uint8).numpy().reshape(t.shape[0], -1)


@pytest.mark.parametrize("n_table,hidden,n_idx,dtype", [
    (1000, 64, 300, torch.float32),
    (5000, 4096, 2048, torch.bfloat16),      # a 7B model's hidden size
    (77, 8, 77, torch.bfloat16),             # one 16-byte piece per row, every row
    (300, 1536, 1, torch.bfloat16),          # a single row
])
def test_rows_match_oracle(n_table, hidden, n_idx, dtype):
    g = torch.Generator().manual_seed(n_table)
    table = torch.randn((n_table, hidden), generator=g).to(dtype)
    idx = torch.sort(torch.randperm(n_table, generator=g)[:n_idx])[0].int()
    print(f"[rows] table={n_table}x{hidden} {dtype} n_idx={n_idx}", flush=True)
    out = binding.reform_gather_rows(table.to(DEV), idx.to(DEV))
    torch.cuda.synchronize()
    want = oracle.gather_rows(raw(table), idx.numpy())
    np.testing.assert_array_equal(raw(out), want)


def test_device_count_and_bad_index_flag():
    g = torch.Generator().manual_seed(1)
    table = torch.randn((500, 128), generator=g).bfloat16()
    idx = torch.tensor([3, 9, 100, 499, 7, 8], dtype=torch.int32)
    count = torch.tensor([4], dtype=torch.int32, device=DEV)
    out = torch.full((6, 128), 5.0, dtype=torch.bfloat16, device=DEV)
    err = torch.zeros((1,), dtype=torch.int32, device=DEV)
    binding.reform_gather_rows(table.to(DEV), idx.to(DEV), count=count, out=out, err=err)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(raw(out[:4]), oracle.gather_rows(raw(table), idx[:4].numpy()))
    assert (out[4:] == 5.0).all() and int(err.item()) == 0              # rows past the count untouched
    bad = torch.tensor([3, 500, -1, 9], dtype=torch.int32, device=DEV)
    out.fill_(5.0)
    binding.reform_gather_rows(table.to(DEV), bad, out=out, err=err)
    torch.cuda.synchronize()
    assert int(err.item()) == 1
    assert (out[1:3] == 5.0).all()                                       # bad rows skipped, never read
    np.testing.assert_array_equal(raw(out[[0, 3]]), oracle.gather_rows(raw(table), np.array([3, 9], np.int32)))


def test_union_of_the_gather_feeds_the_row_gather():
    """reform_gather_topk's union list and its device-side count drive the row gather directly."""
    g = torch.Generator().manual_seed(2)
    N, D, hidden = 30000, 256, 1024
    emb = torch.randn((N, D), generator=g).bfloat16().to(DEV)
    qry = torch.randn((4, D), generator=g).bfloat16().to(DEV)
    table = torch.randn((N, hidden), generator=g).bfloat16()
    _, _, uni, cnt = binding.reform_gather_topk(emb, qry, 512, 8, 16, 16)
    out = torch.zeros((N, hidden), dtype=torch.bfloat16, device=DEV)
    binding.reform_gather_rows(table.to(DEV), uni, count=cnt, out=out)
    torch.cuda.synchronize()
    n = int(cnt.item())
    uni_h = uni.cpu().numpy()[:n]
    np.testing.assert_array_equal(raw(out[:n]), oracle.gather_rows(raw(table), uni_h))
    assert (out[n:] == 0).all()

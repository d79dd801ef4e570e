"""The C-ABI library: loads without a GPU, exports what include/reform.h declares, and rejects
bad descriptors on the host before anything could be launched (no compute call is made here)."""
import ctypes
import os
import re

import pytest

from paper_2506_01215_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    src = open(os.path.join(ROOT, "include", "reform.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(reform_[a-z0-9_]+)\s*\(", src)))


def test_library_exports_every_declared_symbol():
    lib = binding.load_library()
    names = declared_functions()
    assert sorted(names) == sorted(binding.EXPORTED)
    for name in names:
        assert getattr(lib, name) is not None
    assert lib.reform_version() >= 100
    assert lib.reform_status_string(0) == b"ok"


def good_attn():
    return binding.AttnDesc(ctypes.sizeof(binding.AttnDesc), binding.REFORM_BF16, 32, 8, 128,
                            4096, 512, 8192, 512 * 128, 128, 512 * 128, 128, 0.0884, 0, 0, 0)


@pytest.mark.parametrize("field,value,status", [
    ("struct_size", 4, 1), ("dtype", 7, 1), ("n_kv_heads", 5, 1), ("chunk_len", 0, 1),
    ("capacity", 100, 1), ("scale", 0.0, 1), ("scale", float("nan"), 1), ("obs_window", 513, 1),
    ("accumulate", 2, 1), ("phases", 4, 1), ("q_row_stride", 64, 1), ("q_row_stride", 129, 1), ("head_dim", 96, 2),
])
def test_attend_rejects_bad_descriptor(field, value, status):
    lib = binding.load_library()
    d = good_attn()
    if field == "head_dim":
        d.q_row_stride = d.o_row_stride = 96
    setattr(d, field, value)
    assert lib.reform_chunk_attend_score_workspace(ctypes.byref(d)) == 0
    fake = ctypes.c_void_p(0x1000)
    rc = lib.reform_chunk_attend_score(ctypes.byref(d), fake, fake, fake, fake, None, None, None, 0, None)
    assert rc == status


def test_attend_rejects_null_and_missing_workspace():
    lib = binding.load_library()
    d = good_attn()
    assert lib.reform_chunk_attend_score_workspace(ctypes.byref(d)) >= 32 * 512 * 4
    fake = ctypes.c_void_p(0x1000)
    assert lib.reform_chunk_attend_score(ctypes.byref(d), None, fake, fake, fake, None, None, None, 0, None) == 1
    assert lib.reform_chunk_attend_score(ctypes.byref(d), ctypes.c_void_p(0x1004), fake, fake, fake,
                                         None, None, None, 0, None) == 1
    # lse == NULL needs a workspace
    assert lib.reform_chunk_attend_score(ctypes.byref(d), fake, fake, fake, fake, None, None, None, 0, None) == 3
    assert lib.reform_chunk_attend_score(None, fake, fake, fake, fake, None, None, None, 0, None) == 1


def test_evict_rejects_bad_arguments():
    lib = binding.load_library()
    mk = lambda **kw: binding.EvictDesc(**{**dict(struct_size=ctypes.sizeof(binding.EvictDesc),
                                                  dtype=1, n_kv_heads=8, head_dim=128, n_valid=300,
                                                  budget=100, capacity=400, n_sink=0, n_recent=0), **kw})
    fake = ctypes.c_void_p(0x1000)
    call = lambda d, ws=None, n=0: lib.reform_evict_topk_compact(ctypes.byref(d), fake, fake, fake,
                                                                 None, None, ws, n, None)
    assert call(mk(n_valid=500)) == 1
    assert call(mk(n_sink=60, n_recent=60)) == 1
    assert call(mk(budget=0)) == 1
    assert call(mk(struct_size=8)) == 1
    assert call(mk(head_dim=4)) == 2                      # 8-byte rows
    assert call(mk(capacity=(1 << 31) - 1000)) == 2       # index arithmetic needs head room below 2^31
    assert call(mk()) == 3                                # eviction needed but no workspace
    need = lib.reform_evict_topk_compact_workspace(ctypes.byref(mk()))
    assert need >= 8 * 100 * 4 + 2 * 8 * 100 * 4                 # kept indices + score/pos staging
    odd = mk(head_dim=96)                                         # 192-byte rows do not divide 16 KB:
    assert lib.reform_evict_topk_compact_workspace(ctypes.byref(odd)) >= 2 * 8 * 100 * 192   # K/V staging
    assert call(mk(), ctypes.c_void_p(0x1100), need - 1) == 3
    assert call(mk(), ctypes.c_void_p(0x1010), need) == 3  # misaligned


def test_gather_rejects_bad_arguments():
    lib = binding.load_library()
    mk = lambda **kw: binding.GatherDesc(**{**dict(struct_size=ctypes.sizeof(binding.GatherDesc),
                                                   dtype=1, n_ctx=4096, dim=256, n_query=2, k=16,
                                                   radius=0, n_head_keep=0, n_tail_keep=0, eps=1e-8),
                                            **kw})
    fake = ctypes.c_void_p(0x1000)
    call = lambda d, u=None, c=None: lib.reform_gather_topk(ctypes.byref(d), fake, fake, fake, None,
                                                            u, c, None, 0, None)
    assert call(mk(k=0)) == 1
    assert call(mk(k=5000)) == 1
    assert call(mk(eps=0.0)) == 1
    assert call(mk(radius=-1)) == 1
    assert call(mk(dim=100)) == 2
    assert call(mk(n_ctx=1 << 31, k=16)) == 2
    assert call(mk(n_ctx=(1 << 31) - 1000, k=16)) == 2     # index arithmetic needs head room below 2^31
    assert call(mk(), fake, None) == 1                    # union_idx without union_count
    assert call(mk()) == 3                                # no workspace
    assert lib.reform_gather_topk_workspace(ctypes.byref(mk())) >= 2 * 4096 * 4
    assert lib.reform_gather_similarity(ctypes.byref(mk()), fake, fake, None, None) == 1


def test_gather_pooled_rejects_bad_arguments():
    lib = binding.load_library()
    mk = lambda **kw: binding.PooledDesc(**{**dict(struct_size=ctypes.sizeof(binding.PooledDesc),
                                                   dtype=1, n_ctx=4096, dim=256, n_query=2, budget=600,
                                                   pool_window=129, n_head_keep=256, n_tail_keep=256,
                                                   eps=1e-8), **kw})
    fake = ctypes.c_void_p(0x1000)
    call = lambda d, ws=None, nb=0: lib.reform_gather_pooled(ctypes.byref(d), fake, fake, fake, None,
                                                             ws, nb, None)
    assert call(mk(struct_size=8)) == 1
    assert call(mk(budget=0)) == 1
    assert call(mk(budget=5000)) == 1
    assert call(mk(pool_window=128)) == 1                 # even: no centre
    assert call(mk(pool_window=0)) == 1
    assert call(mk(pool_window=1027)) == 2                # beyond the kernel's halo
    assert call(mk(n_head_keep=400, n_tail_keep=256)) == 1   # forced tokens exceed the budget
    assert call(mk(n_tail_keep=-1)) == 1
    assert call(mk(dim=100)) == 2
    assert call(mk()) == 3                                # no workspace
    need = lib.reform_gather_pooled_workspace(ctypes.byref(mk()))
    assert need >= 2 * 4096 * 4 + 4096 * 4                # similarity rows + pooled scores
    assert call(mk(), ctypes.c_void_p(0x1100), need - 1) == 3
    assert lib.reform_gather_pooled_workspace(ctypes.byref(mk(pool_window=2))) == 0


def test_embed_save_rejects_bad_arguments():
    lib = binding.load_library()
    mk = lambda **kw: binding.EmbedDesc(**{**dict(struct_size=ctypes.sizeof(binding.EmbedDesc), dtype=1,
                                                  n_rows=100, head_dim=128, emb_col=256,
                                                  src_row_stride=128, emb_row_stride=2048, eps=1e-12,
                                                  n_heads=1, src_head_stride=0),
                                           **kw})
    fake = ctypes.c_void_p(0x1000)
    call = lambda d, s=fake, e=fake: lib.reform_embed_save_selected(ctypes.byref(d), s, e, None)
    assert call(mk(struct_size=4)) == 1
    assert call(mk(dtype=3)) == 1
    assert call(mk(n_rows=-1)) == 1
    assert call(mk(emb_col=2000)) == 1                    # the segment would overrun the row
    assert call(mk(n_heads=0)) == 1
    assert call(mk(n_heads=15, src_head_stride=12800)) == 1    # 256 + 15 * 128 columns > 2048
    assert call(mk(n_heads=2, src_head_stride=-128)) == 1
    assert call(mk(n_heads=2, src_head_stride=12804)) == 2     # misaligned head stride
    assert call(mk(src_row_stride=64)) == 1               # rows overlap
    assert call(mk(eps=0.0)) == 1
    assert call(mk(), None) == 1
    assert call(mk(head_dim=100, src_row_stride=100)) == 2     # 200-byte rows
    assert call(mk(head_dim=1024, src_row_stride=1024, emb_col=0)) == 2   # 2 KB rows
    assert call(mk(emb_col=4)) == 2                       # misaligned segment
    assert call(mk(), ctypes.c_void_p(0x1008)) == 2       # misaligned source


def test_rerotate_keys_rejects_bad_arguments():
    lib = binding.load_library()
    mk = lambda **kw: binding.RopeDesc(**{**dict(struct_size=ctypes.sizeof(binding.RopeDesc), dtype=1,
                                                 n_kv_heads=8, head_dim=128, capacity=8192, n_rows=4096,
                                                 budget=4096, rotary_dim=128, theta=10000.0), **kw})
    fake = ctypes.c_void_p(0x1000)
    call = lambda d, k=fake, kept=fake: lib.reform_rerotate_keys(ctypes.byref(d), k, kept, None)
    assert call(mk(struct_size=4)) == 1
    assert call(mk(n_rows=5000)) == 1                     # more rows than kept_idx holds
    assert call(mk(rotary_dim=130)) == 1
    assert call(mk(rotary_dim=63)) == 1
    assert call(mk(theta=1.0)) == 1
    assert call(mk(theta=float("inf"))) == 1
    assert call(mk(), fake, None) == 1
    assert call(mk(rotary_dim=8)) == 2                    # half a pair set is not a 16-byte piece
    assert call(mk(), ctypes.c_void_p(0x1004)) == 2


def test_gather_rows_rejects_bad_arguments():
    lib = binding.load_library()
    mk = lambda **kw: binding.RowsDesc(**{**dict(struct_size=ctypes.sizeof(binding.RowsDesc), reserved=0,
                                                 n_table=1000, n_idx=10, row_bytes=256), **kw})
    fake = ctypes.c_void_p(0x1000)
    call = lambda d, t=fake, i=fake, o=fake: lib.reform_gather_rows(ctypes.byref(d), t, i, None, o, None, None)
    assert call(mk(struct_size=4)) == 1
    assert call(mk(reserved=1)) == 1
    assert call(mk(n_table=0)) == 1
    assert call(mk(n_idx=-1)) == 1
    assert call(mk(), None) == 1
    assert call(mk(), fake, None) == 1
    assert call(mk(row_bytes=100)) == 2
    assert call(mk(n_table=1 << 31)) == 2
    assert call(mk(), fake, fake, ctypes.c_void_p(0x1008)) == 2

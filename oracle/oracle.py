"""ctypes/numpy front end of the fp64 CPU oracle (oracle/reform_oracle.c).

TEST INFRASTRUCTURE ONLY.  Argument marshalling and nothing else: every number
is produced by the C file.  Inputs are numpy float32 arrays (bf16 data is
widened to float32 by the caller, which is exact); results are float64/int32.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        path = _build.OUT
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            path = _build.build(force=True)
        lib = ctypes.CDLL(path)
        c_i, c_l, c_d = ctypes.c_int, ctypes.c_int64, ctypes.c_double
        P = ctypes.c_void_p
        lib.oracle_num_threads.restype = c_i
        lib.oracle_set_num_threads.restype = None
        lib.oracle_set_num_threads.argtypes = [c_i]
        lib.oracle_attend_score.restype = c_i
        lib.oracle_attend_score.argtypes = [P, P, P, c_i, c_i, c_i, c_i, c_i, c_i, c_d, c_i, c_i,
                                            P, P, P]
        lib.oracle_attend_rows.restype = c_i
        lib.oracle_attend_rows.argtypes = [P, P, P, c_i, c_i, c_i, c_i, c_i, c_i, c_d, P, P, c_i,
                                           P, P, P]
        lib.oracle_topk_lowest_index.restype = c_i
        lib.oracle_topk_lowest_index.argtypes = [P, c_l, c_l, P]
        lib.oracle_evict_select.restype = c_i
        lib.oracle_evict_select.argtypes = [P, c_i, c_i, c_i, c_i, P]
        lib.oracle_compact_rows.restype = c_i
        lib.oracle_compact_rows.argtypes = [P, P, P, P, c_i, P, c_i]
        lib.oracle_cosine.restype = c_i
        lib.oracle_cosine.argtypes = [P, P, c_l, c_i, c_i, c_d, P]
        lib.oracle_pool_scores.restype = c_i
        lib.oracle_pool_scores.argtypes = [P, c_i, c_l, c_i, P]
        lib.oracle_embed_segment.restype = c_i
        lib.oracle_embed_segment.argtypes = [P, c_l, c_i, c_l, P, c_l, c_l, c_d]
        lib.oracle_rerotate_keys.restype = c_i
        lib.oracle_rerotate_keys.argtypes = [P, P, c_l, c_i, c_i, c_d, P]
        lib.oracle_gather_rows.restype = c_i
        lib.oracle_gather_rows.argtypes = [P, c_l, c_l, P, c_l, P]
        lib.oracle_union_dilate.restype = c_l
        lib.oracle_union_dilate.argtypes = [P, c_i, c_l, c_l, c_i, c_l, c_l, P]
        _LIB = lib
    return _LIB


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads():
    return int(_lib().oracle_num_threads())


def set_num_threads(n):
    """OpenMP thread count for later oracle calls made by the calling thread."""
    _lib().oracle_set_num_threads(int(n))


def attend_score(q, k, v, M, scale, W=0, accumulate=False, score_in=None, want_out=True):
    """q [Hq,Ct,d]; k,v [Hkv,cap,d] with rows [0,M) cache and [M,M+Ct) chunk.

    Returns (out [Hq,Ct,d] f64, lse [Hq,Ct] f64, score [Hkv,cap] f64; entries >= M+Ct are 0).
    """
    q, k, v = _f32(q), _f32(k), _f32(v)
    Hq, Ct, d = q.shape
    Hkv, cap, d2 = k.shape
    assert d2 == d and v.shape == k.shape
    out = np.zeros((Hq, Ct, d), np.float64) if want_out else None
    lse = np.zeros((Hq, Ct), np.float64)
    if accumulate:
        score = np.array(score_in, dtype=np.float64, copy=True, order="C")
        assert score.shape == (Hkv, cap)
    else:
        score = np.zeros((Hkv, cap), np.float64)
    rc = _lib().oracle_attend_score(_ptr(q), _ptr(k), _ptr(v), Hq, Hkv, d, int(M), Ct, cap,
                                    float(scale), int(W), int(bool(accumulate)),
                                    _ptr(out), _ptr(lse), _ptr(score))
    if rc != 0:
        raise ValueError(f"oracle_attend_score rc={rc}")
    return out, lse, score


def attend_rows(q, k, v, M, scale, rows_h, rows_i, want_score=False):
    """Attention output and lse for sampled (head, row) pairs only.

    With want_score, also the attention mass [Hkv,cap] that the SAMPLED rows alone give each key.
    """
    q, k, v = _f32(q), _f32(k), _f32(v)
    Hq, Ct, d = q.shape
    Hkv, cap, _ = k.shape
    rh = np.ascontiguousarray(rows_h, dtype=np.int32)
    ri = np.ascontiguousarray(rows_i, dtype=np.int32)
    n = rh.shape[0]
    out = np.zeros((n, d), np.float64)
    lse = np.zeros((n,), np.float64)
    score = np.zeros((Hkv, cap), np.float64) if want_score else None
    rc = _lib().oracle_attend_rows(_ptr(q), _ptr(k), _ptr(v), Hq, Hkv, d, int(M), Ct, cap,
                                   float(scale), _ptr(rh), _ptr(ri), n, _ptr(out), _ptr(lse),
                                   _ptr(score))
    if rc != 0:
        raise ValueError(f"oracle_attend_rows rc={rc}")
    if want_score:
        return out, lse, score
    return out, lse


def topk_lowest_index(x, keep):
    x = np.ascontiguousarray(x, dtype=np.float64)
    out = np.zeros((int(keep),), np.int32)
    rc = _lib().oracle_topk_lowest_index(_ptr(x), x.shape[0], int(keep), _ptr(out))
    if rc != 0:
        raise ValueError(f"oracle_topk_lowest_index rc={rc}")
    return out


def evict_select(score, n, B, n_sink=0, n_recent=0):
    """score: 1-D (one KV head), first n entries are candidates.  Returns kept idx ascending."""
    s = np.ascontiguousarray(score, dtype=np.float64)
    kept = np.zeros((min(int(n), int(B)),), np.int32)
    rc = _lib().oracle_evict_select(_ptr(s), int(n), int(B), int(n_sink), int(n_recent), _ptr(kept))
    if rc < 0:
        raise ValueError(f"oracle_evict_select rc={rc}")
    assert rc == kept.shape[0]
    return kept


def evict_compact(k, v, score, pos, n, B, n_sink=0, n_recent=0):
    """Per-KV-head retention + order-preserving compaction.

    k, v [Hkv,cap,d] float32; score [Hkv,cap] float64; pos [Hkv,cap] int32 (or None).
    Returns (k2, v2, score2, pos2, kept [Hkv,min(n,B)]); rows >= min(n,B) keep their old content.
    """
    k2 = np.array(k, dtype=np.float32, copy=True, order="C")
    v2 = np.array(v, dtype=np.float32, copy=True, order="C")
    s2 = np.array(score, dtype=np.float64, copy=True, order="C")
    p2 = None if pos is None else np.array(pos, dtype=np.int32, copy=True, order="C")
    Hkv, cap, d = k2.shape
    nk = min(int(n), int(B))
    kept = np.zeros((Hkv, nk), np.int32)
    for g in range(Hkv):
        kept[g] = evict_select(s2[g], n, B, n_sink, n_recent)
        kg = np.ascontiguousarray(kept[g])
        rc = _lib().oracle_compact_rows(_ptr(k2[g]), _ptr(v2[g]), _ptr(s2[g]),
                                        None if p2 is None else _ptr(p2[g]), d, _ptr(kg), nk)
        if rc != 0:
            raise ValueError(f"oracle_compact_rows rc={rc}")
    return k2, v2, s2, p2, kept


def cosine(emb, qry, eps=1e-8):
    emb, qry = _f32(emb), _f32(qry)
    N, D = emb.shape
    nq, D2 = qry.shape
    assert D == D2
    sim = np.zeros((nq, N), np.float64)
    rc = _lib().oracle_cosine(_ptr(emb), _ptr(qry), N, D, nq, float(eps), _ptr(sim))
    if rc != 0:
        raise ValueError(f"oracle_cosine rc={rc}")
    return sim


def union_dilate(topk, N, radius=0, n_head=0, n_tail=0):
    topk = np.ascontiguousarray(topk, dtype=np.int32)
    nq, k = topk.shape
    out = np.zeros((int(N),), np.int32)
    cnt = _lib().oracle_union_dilate(_ptr(topk), nq, k, int(N), int(radius), int(n_head),
                                     int(n_tail), _ptr(out))
    if cnt < 0:
        raise ValueError(f"oracle_union_dilate rc={cnt}")
    return out[:cnt].copy()


def gather(emb, qry, k, radius=0, n_head=0, n_tail=0, eps=1e-8):
    """Full gather: cosine -> per-query top-k (ties to lowest index) -> union with dilation.

    Returns (sim [nq,N] f64, topk [nq,k] i32 ascending, union i32 ascending).
    """
    sim = cosine(emb, qry, eps)
    nq, N = sim.shape
    topk = np.stack([topk_lowest_index(sim[qi], k) for qi in range(nq)])
    return sim, topk, union_dilate(topk, N, radius, n_head, n_tail)


def pool_scores(sim, window):
    """max over the query tokens, then a centred `window`-wide max over adjacent context tokens."""
    sim = np.ascontiguousarray(sim, dtype=np.float64)
    nq, N = sim.shape
    pooled = np.zeros((N,), np.float64)
    rc = _lib().oracle_pool_scores(_ptr(sim), nq, N, int(window), _ptr(pooled))
    if rc != 0:
        raise ValueError(f"oracle_pool_scores rc={rc}")
    return pooled


def gather_pooled(emb, qry, budget, window=129, n_head=0, n_tail=0, eps=1e-8):
    """The paper's own post-processing: cosine -> max over query tokens -> window max-pool ->
    the `budget` highest-scoring tokens, the first n_head and last n_tail always among them
    (ties to the lowest index).  Returns (sim, pooled [N] f64, selected idx ascending)."""
    sim = cosine(emb, qry, eps)
    pooled = pool_scores(sim, window)
    sel = evict_select(pooled, pooled.shape[0], budget, n_head, n_tail)
    return sim, pooled, sel


def embed_segment(src, emb, col, eps=1e-12):
    """src [n_rows, d] float32 (any row stride); emb [n_rows, D] float64, written in place at
    columns [col, col+d): the L2-normalised rows of src."""
    src = np.asarray(src, dtype=np.float32)
    assert src.ndim == 2 and src.strides[1] == 4 and src.strides[0] % 4 == 0
    assert emb.dtype == np.float64 and emb.flags.c_contiguous and emb.shape[0] == src.shape[0]
    rc = _lib().oracle_embed_segment(_ptr(src), src.shape[0], src.shape[1], src.strides[0] // 4,
                                     _ptr(emb), emb.shape[1], int(col), float(eps))
    if rc != 0:
        raise ValueError(f"oracle_embed_segment rc={rc}")
    return emb


def rerotate_keys(k, kept, theta=10000.0, rot=None):
    """k [n_rows, d] float32: one head's compacted key rows; kept [n_rows]: the slot each row came
    from.  Returns the rows rotated by (r - kept[r]) positions, float64."""
    k = _f32(k)
    kept = np.ascontiguousarray(kept, dtype=np.int32)
    n, d = k.shape
    assert kept.shape == (n,)
    out = np.zeros((n, d), np.float64)
    rc = _lib().oracle_rerotate_keys(_ptr(k), _ptr(kept), n, d, d if rot is None else int(rot),
                                     float(theta), _ptr(out))
    if rc != 0:
        raise ValueError(f"oracle_rerotate_keys rc={rc}")
    return out


def gather_rows(table, idx):
    """table [n, ...] any dtype (C-contiguous); idx int32.  Returns table[idx] (raw byte copy)."""
    table = np.ascontiguousarray(table)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    row_bytes = table[0].nbytes if table.shape[0] else int(np.prod(table.shape[1:])) * table.itemsize
    out = np.zeros((idx.shape[0],) + table.shape[1:], table.dtype)
    rc = _lib().oracle_gather_rows(_ptr(table), table.shape[0], row_bytes, _ptr(idx), idx.shape[0], _ptr(out))
    if rc != 0:
        raise ValueError(f"oracle_gather_rows rc={rc}")
    return out

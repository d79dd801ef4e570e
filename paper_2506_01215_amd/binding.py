"""Thin ctypes binding of libreform_hip.so (the C ABI declared in include/reform.h).

Argument marshalling only: torch tensors supply device memory and the current HIP stream;
every step of the path runs in the library's kernels.  There is no fallback: if the shared
library is missing or a call returns a non-OK status, a ReformError is raised.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libreform_hip.so")
_LIB = None

REFORM_F32, REFORM_BF16 = 0, 1
STATUS = {0: "REFORM_OK", 1: "REFORM_ERR_INVALID_ARG", 2: "REFORM_ERR_UNSUPPORTED",
          3: "REFORM_ERR_WORKSPACE", 4: "REFORM_ERR_RUNTIME"}

EXPORTED = [
    "reform_chunk_attend_score_workspace", "reform_chunk_attend_score",
    "reform_evict_topk_compact_workspace", "reform_evict_topk_compact",
    "reform_evict_topk_compact_static", "reform_debug_set_move_spin_limit",
    "reform_gather_topk_workspace", "reform_gather_topk", "reform_gather_similarity",
    "reform_gather_pooled_workspace", "reform_gather_pooled", "reform_embed_save_selected",
    "reform_rerotate_keys", "reform_gather_rows", "reform_probe_mfma_bf16", "reform_probe_stream",
    "reform_status_string", "reform_version",
]


class ReformError(RuntimeError):
    def __init__(self, status, where):
        self.status = int(status)
        super().__init__(f"{where}: {STATUS.get(int(status), status)}")


class AttnDesc(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32),
                ("cache_len", ctypes.c_int32), ("chunk_len", ctypes.c_int32),
                ("capacity", ctypes.c_int32),
                ("q_head_stride", ctypes.c_int64), ("q_row_stride", ctypes.c_int64),
                ("o_head_stride", ctypes.c_int64), ("o_row_stride", ctypes.c_int64),
                ("scale", ctypes.c_float), ("obs_window", ctypes.c_int32),
                ("accumulate", ctypes.c_int32), ("phases", ctypes.c_int32)]


class EvictDesc(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("n_valid", ctypes.c_int32), ("budget", ctypes.c_int32),
                ("capacity", ctypes.c_int32),
                ("n_sink", ctypes.c_int32), ("n_recent", ctypes.c_int32)]


class GatherDesc(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("n_ctx", ctypes.c_int64),
                ("dim", ctypes.c_int32), ("n_query", ctypes.c_int32), ("k", ctypes.c_int32),
                ("radius", ctypes.c_int32), ("n_head_keep", ctypes.c_int32),
                ("n_tail_keep", ctypes.c_int32), ("eps", ctypes.c_float)]


class PooledDesc(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("n_ctx", ctypes.c_int64),
                ("dim", ctypes.c_int32), ("n_query", ctypes.c_int32), ("budget", ctypes.c_int32),
                ("pool_window", ctypes.c_int32), ("n_head_keep", ctypes.c_int32),
                ("n_tail_keep", ctypes.c_int32), ("eps", ctypes.c_float)]


class EmbedDesc(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("n_rows", ctypes.c_int64),
                ("head_dim", ctypes.c_int32), ("emb_col", ctypes.c_int32),
                ("src_row_stride", ctypes.c_int64), ("emb_row_stride", ctypes.c_int64),
                ("eps", ctypes.c_float), ("n_heads", ctypes.c_int32), ("src_head_stride", ctypes.c_int64)]


class RowsDesc(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("reserved", ctypes.c_int32),
                ("n_table", ctypes.c_int64), ("n_idx", ctypes.c_int64), ("row_bytes", ctypes.c_int64)]


class RopeDesc(ctypes.Structure):
    _fields_ = [("struct_size", ctypes.c_uint32), ("dtype", ctypes.c_int32),
                ("n_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("capacity", ctypes.c_int32), ("n_rows", ctypes.c_int32), ("budget", ctypes.c_int32),
                ("rotary_dim", ctypes.c_int32), ("theta", ctypes.c_float)]


def library_path():
    return _LIB_PATH


def load_library():
    """Load libreform_hip.so (built by paper_2506_01215_amd.build); raises if it is absent."""
    global _LIB
    if _LIB is not None:
        return _LIB
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(f"{_LIB_PATH} not found: build it with `python -m paper_2506_01215_amd.build`"
                           " (there is no CPU fallback)")
    lib = ctypes.CDLL(_LIB_PATH)
    vp, sz = ctypes.c_void_p, ctypes.c_size_t
    lib.reform_chunk_attend_score_workspace.restype = sz
    lib.reform_chunk_attend_score_workspace.argtypes = [ctypes.POINTER(AttnDesc)]
    lib.reform_chunk_attend_score.restype = ctypes.c_int
    lib.reform_chunk_attend_score.argtypes = [ctypes.POINTER(AttnDesc), vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.reform_evict_topk_compact_workspace.restype = sz
    lib.reform_evict_topk_compact_workspace.argtypes = [ctypes.POINTER(EvictDesc)]
    lib.reform_evict_topk_compact.restype = ctypes.c_int
    lib.reform_evict_topk_compact.argtypes = [ctypes.POINTER(EvictDesc), vp, vp, vp, vp, vp, vp, sz, vp]
    lib.reform_evict_topk_compact_static.restype = ctypes.c_int
    lib.reform_evict_topk_compact_static.argtypes = [ctypes.POINTER(EvictDesc), vp, vp, vp, vp, vp, vp]
    lib.reform_debug_set_move_spin_limit.restype = None
    lib.reform_debug_set_move_spin_limit.argtypes = [ctypes.c_int32]
    lib.reform_gather_topk_workspace.restype = sz
    lib.reform_gather_topk_workspace.argtypes = [ctypes.POINTER(GatherDesc)]
    lib.reform_gather_topk.restype = ctypes.c_int
    lib.reform_gather_topk.argtypes = [ctypes.POINTER(GatherDesc), vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.reform_gather_similarity.restype = ctypes.c_int
    lib.reform_gather_similarity.argtypes = [ctypes.POINTER(GatherDesc), vp, vp, vp, vp]
    lib.reform_gather_pooled_workspace.restype = sz
    lib.reform_gather_pooled_workspace.argtypes = [ctypes.POINTER(PooledDesc)]
    lib.reform_gather_pooled.restype = ctypes.c_int
    lib.reform_gather_pooled.argtypes = [ctypes.POINTER(PooledDesc), vp, vp, vp, vp, vp, sz, vp]
    lib.reform_embed_save_selected.restype = ctypes.c_int
    lib.reform_embed_save_selected.argtypes = [ctypes.POINTER(EmbedDesc), vp, vp, vp]
    lib.reform_rerotate_keys.restype = ctypes.c_int
    lib.reform_rerotate_keys.argtypes = [ctypes.POINTER(RopeDesc), vp, vp, vp]
    lib.reform_gather_rows.restype = ctypes.c_int
    lib.reform_gather_rows.argtypes = [ctypes.POINTER(RowsDesc), vp, vp, vp, vp, vp, vp]
    lib.reform_probe_mfma_bf16.restype = ctypes.c_int
    lib.reform_probe_mfma_bf16.argtypes = [vp, vp, ctypes.c_int32, ctypes.c_int32, vp]
    lib.reform_probe_stream.restype = ctypes.c_int
    lib.reform_probe_stream.argtypes = [vp, vp, sz, vp, vp]
    lib.reform_status_string.restype = ctypes.c_char_p
    lib.reform_status_string.argtypes = [ctypes.c_int]
    lib.reform_version.restype = ctypes.c_int32
    _LIB = lib
    return lib


def _dtype_code(t):
    if t.dtype == torch.bfloat16:
        return REFORM_BF16
    if t.dtype == torch.float32:
        return REFORM_F32
    raise TypeError(f"unsupported dtype {t.dtype}")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _workspace(nbytes, device, workspace, stream=None):
    if nbytes == 0:
        return None
    if workspace is None:
        workspace = torch.empty(nbytes + 256, dtype=torch.uint8, device=device)
        if stream is not None:
            # a temporary that is dropped on return while the kernels are only enqueued: tell the
            # caching allocator which stream still uses the block
            workspace.record_stream(stream)
    off = (-workspace.data_ptr()) % 256
    ws = workspace[off:]
    return ws


def debug_set_move_spin_limit(polls):
    """Testing aid, see include/reform.h: polls of the in-place move's bounded wait (0 forces the
    give-up branch, a negative value restores the default)."""
    load_library().reform_debug_set_move_spin_limit(int(polls))


def evict_status_word(workspace):
    """The device-side status word of reform_evict_topk_compact (first int32 of the 256-byte
    aligned workspace the caller passed): 0 unless the in-place move's bounded wait expired.
    Reads it back, so it synchronises with the device."""
    off = (-workspace.data_ptr()) % 256
    return int(workspace[off:off + 4].view(torch.int32).item())


def _check(rc, where):
    if rc != 0:
        raise ReformError(rc, where)


# ------------------------------------------------------------------------------------------
def attn_desc(q, k, out, cache_len, scale, obs_window=0, accumulate=False, phases=0):
    Hq, Ct, d = q.shape
    Hkv, cap, d2 = k.shape
    assert d2 == d and q.stride(2) == 1 and out.stride(2) == 1
    return AttnDesc(ctypes.sizeof(AttnDesc), _dtype_code(q), Hq, Hkv, d, int(cache_len), Ct, cap,
                    q.stride(0), q.stride(1), out.stride(0), out.stride(1),
                    float(scale), int(obs_window), int(bool(accumulate)), int(phases))


def reform_chunk_attend_score(q, k, v, cache_len, scale, obs_window=0, accumulate=False,
                              out=None, lse=None, score=None, want_score=True,
                              workspace=None, stream=None, phases=0):
    """q [Hq,Ct,d]; k,v [Hkv,cap,d] (rows [0,M) cache, [M,M+Ct) chunk).  Returns (out, lse, score)."""
    lib = load_library()
    assert k.is_contiguous() and v.is_contiguous() and k.shape == v.shape
    if out is None:
        out = torch.empty_like(q, memory_format=torch.contiguous_format)
    if lse is None:
        lse = torch.empty(q.shape[:2], dtype=torch.float32, device=q.device)
    if score is None and want_score:
        if accumulate:
            raise ValueError("accumulate needs the previous score tensor")
        score = torch.zeros(k.shape[:2], dtype=torch.float32, device=q.device)
    desc = attn_desc(q, k, out, cache_len, scale, obs_window, accumulate, phases)
    need = lib.reform_chunk_attend_score_workspace(ctypes.byref(desc))
    ws = _workspace(need, q.device, workspace, stream)
    rc = lib.reform_chunk_attend_score(ctypes.byref(desc), _ptr(q), _ptr(k), _ptr(v), _ptr(out),
                                       _ptr(lse), _ptr(score), _ptr(ws),
                                       0 if ws is None else ws.numel(), _stream(stream))
    _check(rc, "reform_chunk_attend_score")
    return out, lse, score


def evict_desc(k, n_valid, budget, n_sink=0, n_recent=0):
    Hkv, cap, d = k.shape
    return EvictDesc(ctypes.sizeof(EvictDesc), _dtype_code(k), Hkv, d, int(n_valid), int(budget), cap,
                     int(n_sink), int(n_recent))


def reform_evict_topk_compact(k, v, score, n_valid, budget, n_sink=0, n_recent=0, pos=None,
                              kept_idx=None, workspace=None, stream=None):
    """In-place retention + compaction.  Returns new_len = min(n_valid, budget)."""
    lib = load_library()
    assert k.is_contiguous() and v.is_contiguous() and score.is_contiguous()
    assert score.dtype == torch.float32 and score.shape == k.shape[:2]
    if pos is not None:
        assert pos.dtype == torch.int32 and pos.is_contiguous() and pos.shape == k.shape[:2]
    if kept_idx is not None:
        assert kept_idx.dtype == torch.int32 and kept_idx.is_contiguous()
        assert kept_idx.shape == (k.shape[0], budget)
    desc = evict_desc(k, n_valid, budget, n_sink, n_recent)
    need = lib.reform_evict_topk_compact_workspace(ctypes.byref(desc))
    ws = _workspace(need, k.device, workspace, stream)
    rc = lib.reform_evict_topk_compact(ctypes.byref(desc), _ptr(k), _ptr(v), _ptr(score), _ptr(pos),
                                       _ptr(kept_idx), _ptr(ws), 0 if ws is None else ws.numel(),
                                       _stream(stream))
    _check(rc, "reform_evict_topk_compact")
    return min(int(n_valid), int(budget))


STATIC_SCRATCH_BYTES = 8 << 20


def reform_evict_topk_compact_static(k, v, score, n_valid, budget, n_sink=0, n_recent=0, pos=None,
                                     kept_idx=None, stream=None):
    """reform_evict_topk_compact without a workspace (the library's static device scratch); the
    binding allocates nothing either.  k's device must be the current one."""
    lib = load_library()
    assert k.is_contiguous() and v.is_contiguous() and score.is_contiguous()
    assert score.dtype == torch.float32 and score.shape == k.shape[:2]
    desc = evict_desc(k, n_valid, budget, n_sink, n_recent)
    rc = lib.reform_evict_topk_compact_static(ctypes.byref(desc), _ptr(k), _ptr(v), _ptr(score),
                                              _ptr(pos), _ptr(kept_idx), _stream(stream))
    _check(rc, "reform_evict_topk_compact_static")
    return min(int(n_valid), int(budget))


def gather_desc(emb, qry, k, radius=0, n_head_keep=0, n_tail_keep=0, eps=1e-8):
    N, D = emb.shape
    nq, D2 = qry.shape
    assert D == D2 and emb.dtype == qry.dtype
    return GatherDesc(ctypes.sizeof(GatherDesc), _dtype_code(emb), N, D, nq, int(k), int(radius),
                      int(n_head_keep), int(n_tail_keep), float(eps))


def reform_gather_topk(emb, qry, k, radius=0, n_head_keep=0, n_tail_keep=0, eps=1e-8,
                       want_union=True, topk_idx=None, topk_score=None, union_idx=None,
                       union_count=None, workspace=None, stream=None):
    """Returns (topk_idx [nq,k] i32, topk_score [nq,k] f32, union_idx [N] i32 or None, union_count)."""
    lib = load_library()
    assert emb.is_contiguous() and qry.is_contiguous()
    N, nq = emb.shape[0], qry.shape[0]
    dev = emb.device
    if topk_idx is None:
        topk_idx = torch.empty((nq, k), dtype=torch.int32, device=dev)
    if topk_score is None:
        topk_score = torch.empty((nq, k), dtype=torch.float32, device=dev)
    if want_union:
        if union_idx is None:
            union_idx = torch.empty((N,), dtype=torch.int32, device=dev)
        if union_count is None:
            union_count = torch.zeros((1,), dtype=torch.int32, device=dev)
    desc = gather_desc(emb, qry, k, radius, n_head_keep, n_tail_keep, eps)
    need = lib.reform_gather_topk_workspace(ctypes.byref(desc))
    ws = _workspace(need, dev, workspace, stream)
    rc = lib.reform_gather_topk(ctypes.byref(desc), _ptr(emb), _ptr(qry), _ptr(topk_idx),
                                _ptr(topk_score), _ptr(union_idx), _ptr(union_count), _ptr(ws),
                                0 if ws is None else ws.numel(), _stream(stream))
    _check(rc, "reform_gather_topk")
    return topk_idx, topk_score, union_idx, union_count


def reform_gather_similarity(emb, qry, eps=1e-8, sim=None, stream=None):
    lib = load_library()
    assert emb.is_contiguous() and qry.is_contiguous()
    if sim is None:
        sim = torch.empty((qry.shape[0], emb.shape[0]), dtype=torch.float32, device=emb.device)
    desc = gather_desc(emb, qry, 1, eps=eps)
    rc = lib.reform_gather_similarity(ctypes.byref(desc), _ptr(emb), _ptr(qry), _ptr(sim), _stream(stream))
    _check(rc, "reform_gather_similarity")
    return sim


def reform_embed_save_selected(src, emb, row0, col, eps=1e-12, stream=None):
    """src [n_rows, d] (a view of one head's Q, K or V states; any row stride) or
    [n_heads, n_rows, d] (several heads of one tensor; any head and row strides); writes the
    normalised rows into emb[row0 : row0 + n_rows, col : col + n_heads * d]."""
    lib = load_library()
    if src.dim() == 2:
        src = src.unsqueeze(0)
    nh, n, d = src.shape
    assert nh >= 1 and src.stride(2) == 1 and emb.is_contiguous() and emb.dtype == src.dtype
    assert 0 <= row0 and row0 + n <= emb.shape[0]
    desc = EmbedDesc(ctypes.sizeof(EmbedDesc), _dtype_code(src), n, d, int(col), src.stride(1),
                     emb.shape[1], float(eps), nh, src.stride(0) if nh > 1 else 0)
    dst = emb[row0:] if n else emb
    rc = lib.reform_embed_save_selected(ctypes.byref(desc), _ptr(src), _ptr(dst), _stream(stream))
    _check(rc, "reform_embed_save_selected")
    return emb


def reform_rerotate_keys(k, kept_idx, n_rows, theta=10000.0, rotary_dim=None, stream=None):
    """Rotates the compacted key rows [0, n_rows) of every head in place by (r - kept_idx[r]) positions."""
    lib = load_library()
    assert k.is_contiguous() and kept_idx.is_contiguous() and kept_idx.dtype == torch.int32
    Hkv, cap, d = k.shape
    assert kept_idx.shape[0] == Hkv
    desc = RopeDesc(ctypes.sizeof(RopeDesc), _dtype_code(k), Hkv, d, cap, int(n_rows), kept_idx.shape[1],
                    d if rotary_dim is None else int(rotary_dim), float(theta))
    rc = lib.reform_rerotate_keys(ctypes.byref(desc), _ptr(k), _ptr(kept_idx), _stream(stream))
    _check(rc, "reform_rerotate_keys")
    return k


def reform_gather_rows(table, idx, count=None, out=None, err=None, stream=None):
    """out[i] = table[idx[i]]; `count` (device int32 scalar) limits the rows taken."""
    lib = load_library()
    assert table.is_contiguous() and idx.is_contiguous() and idx.dtype == torch.int32 and idx.dim() == 1
    row_bytes = table[0].numel() * table.element_size()
    if out is None:
        out = torch.empty((idx.shape[0],) + tuple(table.shape[1:]), dtype=table.dtype, device=table.device)
    assert out.is_contiguous() and out.shape[0] >= idx.shape[0]
    desc = RowsDesc(ctypes.sizeof(RowsDesc), 0, table.shape[0], idx.shape[0], row_bytes)
    rc = lib.reform_gather_rows(ctypes.byref(desc), _ptr(table), _ptr(idx), _ptr(count), _ptr(out),
                                _ptr(err), _stream(stream))
    _check(rc, "reform_gather_rows")
    return out


def pooled_desc(emb, qry, budget, pool_window=129, n_head_keep=0, n_tail_keep=0, eps=1e-8):
    N, D = emb.shape
    nq, D2 = qry.shape
    assert D == D2 and emb.dtype == qry.dtype
    return PooledDesc(ctypes.sizeof(PooledDesc), _dtype_code(emb), N, D, nq, int(budget),
                      int(pool_window), int(n_head_keep), int(n_tail_keep), float(eps))


def reform_gather_pooled(emb, qry, budget, pool_window=129, n_head_keep=0, n_tail_keep=0, eps=1e-8,
                         sel_idx=None, pooled=None, workspace=None, stream=None):
    """Returns (sel_idx [budget] i32 ascending, pooled [N] f32)."""
    lib = load_library()
    assert emb.is_contiguous() and qry.is_contiguous()
    dev = emb.device
    if sel_idx is None:
        sel_idx = torch.empty((budget,), dtype=torch.int32, device=dev)
    if pooled is None:
        pooled = torch.empty((emb.shape[0],), dtype=torch.float32, device=dev)
    desc = pooled_desc(emb, qry, budget, pool_window, n_head_keep, n_tail_keep, eps)
    need = lib.reform_gather_pooled_workspace(ctypes.byref(desc))
    ws = _workspace(need, dev, workspace, stream)
    rc = lib.reform_gather_pooled(ctypes.byref(desc), _ptr(emb), _ptr(qry), _ptr(sel_idx), _ptr(pooled),
                                  _ptr(ws), 0 if ws is None else ws.numel(), _stream(stream))
    _check(rc, "reform_gather_pooled")
    return sel_idx, pooled


def pooled_workspace_bytes(desc):
    return load_library().reform_gather_pooled_workspace(ctypes.byref(desc))


def attend_workspace_bytes(desc):
    return load_library().reform_chunk_attend_score_workspace(ctypes.byref(desc))


def evict_workspace_bytes(desc):
    return load_library().reform_evict_topk_compact_workspace(ctypes.byref(desc))


def gather_workspace_bytes(desc):
    return load_library().reform_gather_topk_workspace(ctypes.byref(desc))


def probe_mfma_bf16(operands, sink, iters, workgroups, stream=None):
    """Measurement aid: a pure bf16 MFMA loop; returns the flop it executes."""
    assert operands.numel() * operands.element_size() >= 65536 and sink.numel() * sink.element_size() >= 16
    rc = load_library().reform_probe_mfma_bf16(_ptr(operands), _ptr(sink), int(iters), int(workgroups),
                                               _stream(stream))
    _check(rc, "reform_probe_mfma_bf16")
    return float(workgroups) * 8 * iters * 16 * 16384


def probe_stream(src, dst, sink, stream=None):
    """Measurement aid: read src (and copy it to dst unless dst is None); returns the bytes moved."""
    nbytes = src.numel() * src.element_size()
    assert src.is_contiguous() and (dst is None or (dst.is_contiguous() and dst.numel() * dst.element_size() >= nbytes))
    rc = load_library().reform_probe_stream(_ptr(src), _ptr(dst), nbytes, _ptr(sink), _stream(stream))
    _check(rc, "reform_probe_stream")
    return float(nbytes) * (1 if dst is None else 2)

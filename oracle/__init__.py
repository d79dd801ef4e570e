"""CPU oracle for the REFORM compress-and-gather hot path.

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py.  The GPU library and its Python binding never
import this package, and this package imports nothing from them.
"""
from .oracle import (  # noqa: F401
    attend_score, attend_rows, topk_lowest_index, evict_select, evict_compact,
    cosine, gather, union_dilate, num_threads, set_num_threads, pool_scores, gather_pooled, embed_segment, rerotate_keys, gather_rows,
)

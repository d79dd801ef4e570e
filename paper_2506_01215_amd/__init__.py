"""MI355X-native REFORM compress-and-gather hot path (arXiv 2506.01215).

`binding` exposes the C-ABI library's calls (same names as include/reform.h);
`synth` draws the seeded synthetic workloads.  The native library is loaded on
first use and its absence is an error: there is no CPU fallback.
"""
from . import synth  # noqa: F401
from . import binding  # noqa: F401
from .binding import (  # noqa: F401
    ReformError, load_library, library_path,
    reform_chunk_attend_score, reform_evict_topk_compact, reform_gather_topk,
)

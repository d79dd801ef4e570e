# placeholder replaced below
class ReformError(RuntimeError):
    pass
def load_library(): raise ReformError("not built")
def library_path(): return ""
def reform_chunk_attend_score(*a, **k): raise ReformError("not built")
def reform_evict_topk_compact(*a, **k): raise ReformError("not built")
def reform_gather_topk(*a, **k): raise ReformError("not built")

// C ABI of the library (see include/reform.h): host-side validation, workspace carving and
// kernel launches.  Nothing here allocates device memory or synchronises.
#include "../../include/reform.h"
#include "common.h"

#include <atomic>
#include <cmath>
#include <cstring>

namespace reform {
hipError_t attend_bf16_forward(const AttnParams &p, hipStream_t st);
hipError_t attend_bf16_score(const AttnParams &p, hipStream_t st);
hipError_t attend_f32_forward(const AttnParams &p, hipStream_t st);
hipError_t attend_f32_score(const AttnParams &p, hipStream_t st);

hipError_t evict_run(const EvictParams &p, hipStream_t st);
hipError_t evict_fill_identity(int32_t *kept, int Hkv, int B, int n, hipStream_t st);

hipError_t gather_similarity(GatherParams p, int dtype_is_bf16, hipStream_t st);
hipError_t gather_select_union(GatherParams p, hipStream_t st);
hipError_t gather_pool_select(const PoolParams &p, hipStream_t st);
int gather_pool_max_window();
hipError_t embed_save(const EmbedParams &p, bool bf16, hipStream_t st);
hipError_t rope_rerotate_launch(const RopeParams &p, bool bf16, hipStream_t st);
hipError_t gather_rows_launch(const RowsParams &p, hipStream_t st);
hipError_t probe_mfma_launch(const void *operands, float *sink, int iters, int workgroups, hipStream_t st);
hipError_t probe_stream_launch(const void *src, void *dst, size_t bytes, void *sink, hipStream_t st);
}  // namespace reform

using namespace reform;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }
inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }
inline size_t elt_size(int dtype) { return dtype == REFORM_BF16 ? 2 : 4; }

reform_status check_attn(const reform_attn_desc *d)
{
    if (!d || d->struct_size != sizeof(reform_attn_desc)) return REFORM_ERR_INVALID_ARG;
    if (d->dtype != REFORM_F32 && d->dtype != REFORM_BF16) return REFORM_ERR_INVALID_ARG;
    if (d->n_q_heads <= 0 || d->n_kv_heads <= 0 || d->n_q_heads % d->n_kv_heads) return REFORM_ERR_INVALID_ARG;
    if (d->head_dim <= 0 || d->cache_len < 0 || d->chunk_len <= 0) return REFORM_ERR_INVALID_ARG;
    if ((int64_t)d->cache_len + d->chunk_len > d->capacity) return REFORM_ERR_INVALID_ARG;
    if (!(d->scale > 0.f) || !std::isfinite(d->scale)) return REFORM_ERR_INVALID_ARG;
    if (d->obs_window < 0 || d->obs_window > d->chunk_len) return REFORM_ERR_INVALID_ARG;
    if (d->accumulate != 0 && d->accumulate != 1) return REFORM_ERR_INVALID_ARG;
    if (d->phases < 0 || d->phases > 3) return REFORM_ERR_INVALID_ARG;
    if (d->q_row_stride < d->head_dim || d->o_row_stride < d->head_dim) return REFORM_ERR_INVALID_ARG;
    if (d->q_head_stride < 0 || d->o_head_stride < 0) return REFORM_ERR_INVALID_ARG;
    const int per16 = (int)(16 / elt_size(d->dtype));
    if (d->q_row_stride % per16 || d->q_head_stride % per16 || d->o_row_stride % per16 ||
        d->o_head_stride % per16)
        return REFORM_ERR_INVALID_ARG;
    if (d->dtype == REFORM_BF16) {
        if (d->head_dim != 64 && d->head_dim != 128) return REFORM_ERR_UNSUPPORTED;
    } else {
        if (d->head_dim % 4 || d->head_dim > 256) return REFORM_ERR_UNSUPPORTED;
    }
    if ((int64_t)d->n_q_heads * d->chunk_len >= (1ll << 31) ||
        (int64_t)d->n_kv_heads * ((int64_t)d->cache_len + d->chunk_len) >= (1ll << 31))
        return REFORM_ERR_UNSUPPORTED;
    return REFORM_OK;
}

reform_status check_evict(const reform_evict_desc *d)
{
    if (!d || d->struct_size != sizeof(reform_evict_desc)) return REFORM_ERR_INVALID_ARG;
    if (d->dtype != REFORM_F32 && d->dtype != REFORM_BF16) return REFORM_ERR_INVALID_ARG;
    if (d->n_kv_heads <= 0 || d->head_dim <= 0) return REFORM_ERR_INVALID_ARG;
    if (d->n_valid < 0 || d->budget <= 0 || d->n_valid > d->capacity) return REFORM_ERR_INVALID_ARG;
    if (d->n_sink < 0 || d->n_recent < 0 || (int64_t)d->n_sink + d->n_recent > d->budget)
        return REFORM_ERR_INVALID_ARG;
    if ((d->head_dim * elt_size(d->dtype)) % 16) return REFORM_ERR_UNSUPPORTED;
    if (d->n_kv_heads > 65535) return REFORM_ERR_UNSUPPORTED;
    if ((int64_t)d->capacity > (1ll << 31) - 65536) return REFORM_ERR_UNSUPPORTED;   // room for tile overhang in int32
    return REFORM_OK;
}

reform_status check_gather(const reform_gather_desc *d)
{
    if (!d || d->struct_size != sizeof(reform_gather_desc)) return REFORM_ERR_INVALID_ARG;
    if (d->dtype != REFORM_F32 && d->dtype != REFORM_BF16) return REFORM_ERR_INVALID_ARG;
    if (d->n_ctx <= 0 || d->dim <= 0 || d->n_query <= 0) return REFORM_ERR_INVALID_ARG;
    if (d->k <= 0 || d->k > d->n_ctx) return REFORM_ERR_INVALID_ARG;
    if (d->radius < 0 || d->n_head_keep < 0 || d->n_tail_keep < 0) return REFORM_ERR_INVALID_ARG;
    if (!(d->eps > 0.f) || !std::isfinite(d->eps)) return REFORM_ERR_INVALID_ARG;
    if (d->n_ctx > (1ll << 31) - 65536) return REFORM_ERR_UNSUPPORTED;   // int32 indices, with room for tile overhang
    if (d->dim % 8) return REFORM_ERR_UNSUPPORTED;
    if (d->n_query > 65535) return REFORM_ERR_UNSUPPORTED;
    const int grp = d->n_query < 16 ? d->n_query : 16;
    if ((size_t)grp * d->dim * 4 > 150 * 1024 && !(d->dtype == REFORM_BF16 && d->dim % 32 == 0 &&
                                                     (size_t)16 * (d->dim + 128) * 2 <= 150 * 1024))
        return REFORM_ERR_UNSUPPORTED;
    return REFORM_OK;
}

// Row pitch (floats) of the similarity rows inside the workspace: a multiple of 16 bytes for any
// n_ctx, so that the similarity kernel can store and the selection can load 16-byte quads, and
// skewed by 4352 bytes so that the query rows a wave writes at once do not sit a power of two
// apart (at 2^20 rows the whole gather call measured 4 % slower without the skew; skews from 256 B
// to 64 KB measured alike).
long sim_pitch(int64_t n_ctx) { return (long)((n_ctx + 63) / 64 * 64 + 1088); }

struct GatherLayout {
    size_t sim, hist, prefix, krem, blk, bitmap, words, total;
    int nblk, nwords, nublk;
};

GatherLayout gather_layout(const reform_gather_desc *d)
{
    GatherLayout L;
    L.nblk = (int)((d->n_ctx + 4095) / 4096);
    L.nwords = (int)((d->n_ctx + 31) / 32);
    L.nublk = (L.nwords + kUnionWordsPerBlock - 1) / kUnionWordsPerBlock;
    size_t off = 0;
    L.sim = off;    off += align_up((size_t)d->n_query * sim_pitch(d->n_ctx) * sizeof(float));
    L.hist = off;   off += align_up((size_t)d->n_query * 3 * 2048 * sizeof(int));
    L.prefix = off; off += align_up((size_t)3 * d->n_query * sizeof(uint32_t));
    L.krem = off;   off += align_up((size_t)3 * d->n_query * sizeof(int));
    L.blk = off;    off += align_up((size_t)d->n_query * L.nblk * 2 * sizeof(int));
    L.bitmap = off; off += align_up((size_t)L.nwords * sizeof(uint32_t));
    L.words = off;  off += align_up((size_t)L.nublk * sizeof(int));
    L.total = off;
    return L;
}

reform_gather_desc pooled_as_gather(const reform_pooled_desc *d)
{
    reform_gather_desc g;
    std::memset(&g, 0, sizeof(g));
    g.struct_size = sizeof(g);
    g.dtype = d->dtype; g.n_ctx = d->n_ctx; g.dim = d->dim; g.n_query = d->n_query;
    g.k = d->budget; g.eps = d->eps;
    return g;
}

reform_status check_pooled(const reform_pooled_desc *d)
{
    if (!d || d->struct_size != sizeof(reform_pooled_desc)) return REFORM_ERR_INVALID_ARG;
    const reform_gather_desc g = pooled_as_gather(d);
    const reform_status rc = check_gather(&g);
    if (rc != REFORM_OK) return rc;
    if (d->pool_window < 1 || (d->pool_window % 2) == 0) return REFORM_ERR_INVALID_ARG;
    if (d->n_head_keep < 0 || d->n_tail_keep < 0 ||
        (int64_t)d->n_head_keep + d->n_tail_keep > d->budget)
        return REFORM_ERR_INVALID_ARG;
    if (d->pool_window > gather_pool_max_window()) return REFORM_ERR_UNSUPPORTED;
    return REFORM_OK;
}

struct PooledLayout {
    size_t status, sim, pooled, hist, prefix, krem, blk, total;
    int nblk;
};

PooledLayout pooled_layout(const reform_pooled_desc *d)
{
    PooledLayout L;
    L.nblk = (int)((d->n_ctx + 4095) / 4096);
    size_t off = 0;
    L.status = off; off += align_up(sizeof(int));
    L.sim = off;    off += align_up((size_t)d->n_query * sim_pitch(d->n_ctx) * sizeof(float));
    L.pooled = off; off += align_up((size_t)d->n_ctx * sizeof(float));
    L.hist = off;   off += align_up((size_t)3 * 2048 * sizeof(int));
    L.prefix = off; off += align_up((size_t)3 * sizeof(uint32_t));
    L.krem = off;   off += align_up((size_t)3 * sizeof(int));
    L.blk = off;    off += align_up((size_t)L.nblk * 2 * sizeof(int));
    L.total = off;
    return L;
}

}  // namespace

extern "C" {

const char *reform_status_string(reform_status s)
{
    switch (s) {
    case REFORM_OK: return "ok";
    case REFORM_ERR_INVALID_ARG: return "invalid argument";
    case REFORM_ERR_UNSUPPORTED: return "unsupported shape or type";
    case REFORM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case REFORM_ERR_RUNTIME: return "HIP runtime error";
    }
    return "unknown status";
}

int32_t reform_version(void) { return 100; }

// ---------------------------------------------------------------------------------------
size_t reform_chunk_attend_score_workspace(const reform_attn_desc *d)
{
    if (check_attn(d) != REFORM_OK) return 0;
    return align_up((size_t)d->n_q_heads * d->chunk_len * sizeof(float));
}

reform_status reform_chunk_attend_score(const reform_attn_desc *d, const void *q, const void *k,
                                        const void *v, void *out, float *lse, float *score,
                                        void *workspace, size_t workspace_bytes, void *hip_stream)
{
    reform_status rc = check_attn(d);
    if (rc != REFORM_OK) return rc;
    const bool do_attn = d->phases != 2, do_score = d->phases != 1 && score != nullptr;
    if (!q || !k || !v || (do_attn && !out)) return REFORM_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(v) || !aligned16(out)) return REFORM_ERR_INVALID_ARG;
    if (d->phases == 2 && (!lse || !score)) return REFORM_ERR_INVALID_ARG;
    float *lse_buf = lse;
    if (!lse_buf) {
        const size_t need = reform_chunk_attend_score_workspace(d);
        if (!workspace || workspace_bytes < need || ((uintptr_t)workspace & (kAlign - 1)))
            return REFORM_ERR_WORKSPACE;
        lse_buf = (float *)workspace;
    }
    AttnParams p;
    std::memset(&p, 0, sizeof(p));
    p.q = q; p.k = k; p.v = v; p.out = out; p.lse = lse_buf; p.score = score;
    p.Hq = d->n_q_heads; p.Hkv = d->n_kv_heads; p.G = p.Hq / p.Hkv; p.D = d->head_dim;
    p.M = d->cache_len; p.Ct = d->chunk_len; p.cap = d->capacity; p.n = p.M + p.Ct;
    p.q_hs = d->q_head_stride; p.q_rs = d->q_row_stride;
    p.o_hs = d->o_head_stride; p.o_rs = d->o_row_stride;
    p.scale = d->scale;
    p.W = d->obs_window ? d->obs_window : d->chunk_len;
    p.accumulate = d->accumulate;
    hipStream_t st = (hipStream_t)hip_stream;
    hipError_t e = hipSuccess;
    if (d->dtype == REFORM_BF16) {
        if (do_attn) e = attend_bf16_forward(p, st);
        if (e == hipSuccess && do_score) e = attend_bf16_score(p, st);
    } else {
        if (do_attn) e = attend_f32_forward(p, st);
        if (e == hipSuccess && do_score) e = attend_f32_score(p, st);
    }
    return e == hipSuccess ? REFORM_OK : REFORM_ERR_RUNTIME;
}

// ---------------------------------------------------------------------------------------
// Polls of the in-place move's bounded wait (see reform_debug_set_move_spin_limit).
static std::atomic<int> g_move_spin_limit{1 << 22};

void reform_debug_set_move_spin_limit(int32_t polls)
{
    g_move_spin_limit.store(polls < 0 ? (1 << 22) : polls, std::memory_order_relaxed);
}

struct EvictLayout {
    size_t kept, stage_k, stage_v, stage_score, stage_pos, hist, prefix, krem, blk, sync, rank, total;
    int nblk, ntile;
    bool inplace;
};

static EvictLayout evict_layout(const reform_evict_desc *d)
{
    EvictLayout L;
    const size_t rows = (size_t)d->n_kv_heads * d->budget;
    const size_t row_bytes = (size_t)d->head_dim * elt_size(d->dtype);
    L.nblk = (d->n_valid + 4095) / 4096;
    size_t off = 0;
    // rows whose size divides 16 KB move in place; other sizes go through K/V staging
    L.inplace = row_bytes <= (size_t)kMoveTileBytes && ((size_t)kMoveTileBytes % row_bytes) == 0;
    L.ntile = L.inplace ? (int)(((size_t)d->budget * row_bytes + kMoveTileBytes - 1) / kMoveTileBytes) : 0;
    // the synchronisation words of the in-place move come first: word 0 of the workspace is its
    // error word (documented in the header), then the per-stream tickets and the per-tile flags
    L.sync = off;        off += align_up((size_t)(32 * (1 + 2 * d->n_kv_heads) + 2 * d->n_kv_heads * (L.ntile ? L.ntile : 1)) * sizeof(int));
    L.kept = off;        off += align_up(rows * sizeof(int32_t));
    L.stage_k = off;     off += L.inplace ? 0 : align_up(rows * row_bytes);
    L.stage_v = off;     off += L.inplace ? 0 : align_up(rows * row_bytes);
    L.stage_score = off; off += align_up(rows * sizeof(float));
    L.stage_pos = off;   off += align_up(rows * sizeof(int32_t));
    L.hist = off;        off += align_up((size_t)d->n_kv_heads * 3 * 2048 * sizeof(int));
    L.prefix = off;      off += align_up((size_t)3 * d->n_kv_heads * sizeof(uint32_t));
    L.krem = off;        off += align_up((size_t)3 * d->n_kv_heads * sizeof(int));
    L.blk = off;         off += align_up((size_t)d->n_kv_heads * (L.nblk ? L.nblk : 1) * 2 * sizeof(int));
    L.rank = off;        off += L.inplace ? align_up((size_t)d->n_kv_heads * d->capacity * sizeof(int32_t)) : 0;
    L.total = off;
    return L;
}

size_t reform_evict_topk_compact_workspace(const reform_evict_desc *d)
{
    if (check_evict(d) != REFORM_OK) return 0;
    return evict_layout(d).total;
}

reform_status reform_evict_topk_compact(const reform_evict_desc *d, void *k, void *v, float *score,
                                        int32_t *pos, int32_t *kept_idx, void *workspace,
                                        size_t workspace_bytes, void *hip_stream)
{
    reform_status rc = check_evict(d);
    if (rc != REFORM_OK) return rc;
    if (!k || !v || !score) return REFORM_ERR_INVALID_ARG;
    if (!aligned16(k) || !aligned16(v)) return REFORM_ERR_INVALID_ARG;
    hipStream_t st = (hipStream_t)hip_stream;
    if (d->n_valid <= d->budget) {   // nothing to evict: new_len = n_valid, no data moves
        if (kept_idx && evict_fill_identity(kept_idx, d->n_kv_heads, d->budget, d->n_valid, st) != hipSuccess)
            return REFORM_ERR_RUNTIME;
        return REFORM_OK;
    }
    const EvictLayout L = evict_layout(d);
    if (!workspace || workspace_bytes < L.total || ((uintptr_t)workspace & (kAlign - 1)))
        return REFORM_ERR_WORKSPACE;
    char *ws = (char *)workspace;
    EvictParams p;
    std::memset(&p, 0, sizeof(p));
    p.k = k; p.v = v; p.score = score; p.pos = pos;
    p.kept = kept_idx ? kept_idx : (int32_t *)(ws + L.kept);
    p.stage_k = ws + L.stage_k;
    p.stage_v = ws + L.stage_v;
    p.stage_score = (float *)(ws + L.stage_score);
    p.stage_pos = (int32_t *)(ws + L.stage_pos);
    p.Hkv = d->n_kv_heads; p.n = d->n_valid; p.B = d->budget; p.cap = d->capacity;
    p.n_sink = d->n_sink; p.n_recent = d->n_recent;
    p.row_bytes = (int)(d->head_dim * elt_size(d->dtype));
    p.sel.vals = score; p.sel.ld = d->capacity; p.sel.N = d->n_valid;
    p.sel.nq = d->n_kv_heads; p.sel.k = d->budget;
    p.sel.n_sink = d->n_sink; p.sel.n_recent = d->n_recent;
    p.sel.hist = (int *)(ws + L.hist);
    p.sel.sel_prefix = (uint32_t *)(ws + L.prefix);
    p.sel.sel_krem = (int *)(ws + L.krem);
    p.sel.blk_cnt = (int *)(ws + L.blk);
    p.sel.nblk = L.nblk;
    p.sel.out_idx = p.kept; p.sel.out_val = nullptr; p.sel.out_ld = d->budget;
    p.sel.out_rank = L.inplace ? (int32_t *)(ws + L.rank) : nullptr;
    p.sel.multi_ok = 1;
    p.sel.spin_limit = g_move_spin_limit.load(std::memory_order_relaxed);
    p.sync = L.inplace ? (int *)(ws + L.sync) : nullptr;
    p.ntile = L.ntile;
    p.spin_limit = g_move_spin_limit.load(std::memory_order_relaxed);
    return evict_run(p, st) == hipSuccess ? REFORM_OK : REFORM_ERR_RUNTIME;
}

// ---------------------------------------------------------------------------------------
// The same call for callers that cannot allocate: the workspace is a static device array that
// every GPU the library runs on holds until the process ends.  `static_scratch` is only a
// host-side stand-in for the symbol; the device address is looked up once per device with that
// device current and only that address is ever handed to a kernel.
}  // extern "C"

static __device__ __align__(256) unsigned char static_scratch[REFORM_STATIC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void *> g_static_scratch_ptr[kMaxDevices];

// Device address of static_scratch on the current device (nullptr on failure).  Two threads
// racing here look up the same address, so the plain atomic store is enough.
void *static_scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *ptr = g_static_scratch_ptr[dev].load(std::memory_order_acquire);
    if (ptr) return ptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(static_scratch)) != hipSuccess || !ptr) return nullptr;
    g_static_scratch_ptr[dev].store(ptr, std::memory_order_release);
    return ptr;
}
}  // namespace

extern "C" {

reform_status reform_evict_topk_compact_static(const reform_evict_desc *d, void *k, void *v,
                                               float *score, int32_t *pos, int32_t *kept_idx,
                                               void *hip_stream)
{
    const reform_status rc = check_evict(d);
    if (rc != REFORM_OK) return rc;
    if (d->n_valid <= d->budget)               // nothing is evicted: no scratch is touched
        return reform_evict_topk_compact(d, k, v, score, pos, kept_idx, nullptr, 0, hip_stream);
    if (evict_layout(d).total > (size_t)REFORM_STATIC_SCRATCH_BYTES) return REFORM_ERR_WORKSPACE;
    void *ws = static_scratch_on_current_device();
    if (!ws) return REFORM_ERR_RUNTIME;
    return reform_evict_topk_compact(d, k, v, score, pos, kept_idx, ws,
                                     (size_t)REFORM_STATIC_SCRATCH_BYTES, hip_stream);
}

// ---------------------------------------------------------------------------------------
size_t reform_gather_topk_workspace(const reform_gather_desc *d)
{
    if (check_gather(d) != REFORM_OK) return 0;
    return gather_layout(d).total;
}

static void fill_gather(GatherParams &p, const reform_gather_desc *d, const void *emb, const void *qry)
{
    std::memset(&p, 0, sizeof(p));
    p.emb = emb; p.qry = qry;
    p.N = d->n_ctx; p.D = d->dim; p.nq = d->n_query; p.k = d->k;
    p.radius = d->radius; p.n_head = d->n_head_keep; p.n_tail = d->n_tail_keep;
    p.eps = d->eps;
}

reform_status reform_gather_similarity(const reform_gather_desc *d, const void *emb, const void *qry,
                                       float *sim, void *hip_stream)
{
    reform_status rc = check_gather(d);
    if (rc != REFORM_OK) return rc;
    if (!emb || !qry || !sim || !aligned16(emb) || !aligned16(qry)) return REFORM_ERR_INVALID_ARG;
    GatherParams p;
    fill_gather(p, d, emb, qry);
    p.sim = sim;
    p.sim_ld = d->n_ctx;                          // the caller's matrix is dense
    return gather_similarity(p, d->dtype == REFORM_BF16, (hipStream_t)hip_stream) == hipSuccess
               ? REFORM_OK : REFORM_ERR_RUNTIME;
}

reform_status reform_gather_topk(const reform_gather_desc *d, const void *emb, const void *qry,
                                 int32_t *topk_idx, float *topk_score, int32_t *union_idx,
                                 int32_t *union_count, void *workspace, size_t workspace_bytes,
                                 void *hip_stream)
{
    reform_status rc = check_gather(d);
    if (rc != REFORM_OK) return rc;
    if (!emb || !qry || !topk_idx || !aligned16(emb) || !aligned16(qry)) return REFORM_ERR_INVALID_ARG;
    if ((union_idx != nullptr) != (union_count != nullptr)) return REFORM_ERR_INVALID_ARG;
    const GatherLayout L = gather_layout(d);
    if (!workspace || workspace_bytes < L.total || ((uintptr_t)workspace & (kAlign - 1)))
        return REFORM_ERR_WORKSPACE;
    char *ws = (char *)workspace;
    GatherParams p;
    fill_gather(p, d, emb, qry);
    p.sim = (float *)(ws + L.sim);
    p.sim_ld = sim_pitch(d->n_ctx);
    p.topk_idx = topk_idx; p.topk_score = topk_score;
    p.union_idx = union_idx; p.union_count = union_count;
    p.bitmap = (uint32_t *)(ws + L.bitmap);
    p.word_cnt = (int *)(ws + L.words);
    p.nwords = L.nwords;
    p.sel.vals = p.sim; p.sel.ld = p.sim_ld; p.sel.N = d->n_ctx;
    p.sel.nq = d->n_query; p.sel.k = d->k;
    p.sel.n_sink = 0; p.sel.n_recent = 0;
    p.sel.hist = (int *)(ws + L.hist);
    p.sel.sel_prefix = (uint32_t *)(ws + L.prefix);
    p.sel.sel_krem = (int *)(ws + L.krem);
    p.sel.blk_cnt = (int *)(ws + L.blk);
    p.sel.nblk = L.nblk;
    p.sel.out_idx = topk_idx; p.sel.out_val = topk_score; p.sel.out_ld = d->k;
    if (union_idx) {                          // the bitmap is cleared together with the histograms ...
        p.sel.zero_extra = (int *)p.bitmap;
        p.sel.zero_extra_n = L.nwords;
    }
    p.sel.pre_zeroed = 1;                     // ... by the first similarity launch
    hipStream_t st = (hipStream_t)hip_stream;
    if (gather_similarity(p, d->dtype == REFORM_BF16, st) != hipSuccess) return REFORM_ERR_RUNTIME;
    return gather_select_union(p, st) == hipSuccess ? REFORM_OK : REFORM_ERR_RUNTIME;
}

// ---------------------------------------------------------------------------------------
size_t reform_gather_pooled_workspace(const reform_pooled_desc *d)
{
    if (check_pooled(d) != REFORM_OK) return 0;
    return pooled_layout(d).total;
}

reform_status reform_gather_pooled(const reform_pooled_desc *d, const void *emb, const void *qry,
                                   int32_t *sel_idx, float *pooled, void *workspace,
                                   size_t workspace_bytes, void *hip_stream)
{
    reform_status rc = check_pooled(d);
    if (rc != REFORM_OK) return rc;
    if (!emb || !qry || !sel_idx || !aligned16(emb) || !aligned16(qry)) return REFORM_ERR_INVALID_ARG;
    const PooledLayout L = pooled_layout(d);
    if (!workspace || workspace_bytes < L.total || ((uintptr_t)workspace & (kAlign - 1)))
        return REFORM_ERR_WORKSPACE;
    char *ws = (char *)workspace;
    hipStream_t st = (hipStream_t)hip_stream;
    const reform_gather_desc g = pooled_as_gather(d);
    GatherParams gp;
    fill_gather(gp, &g, emb, qry);
    gp.sim = (float *)(ws + L.sim);
    gp.sim_ld = sim_pitch(d->n_ctx);
    if (gather_similarity(gp, d->dtype == REFORM_BF16, st) != hipSuccess) return REFORM_ERR_RUNTIME;
    PoolParams p;
    std::memset(&p, 0, sizeof(p));
    p.sim = gp.sim;
    p.pooled = pooled ? pooled : (float *)(ws + L.pooled);
    p.N = d->n_ctx; p.ld = gp.sim_ld; p.nq = d->n_query; p.window = d->pool_window;
    p.sel.vals = p.pooled; p.sel.ld = d->n_ctx; p.sel.N = d->n_ctx;
    p.sel.nq = 1; p.sel.k = d->budget;
    p.sel.n_sink = d->n_head_keep; p.sel.n_recent = d->n_tail_keep;
    p.sel.hist = (int *)(ws + L.hist);
    p.sel.sel_prefix = (uint32_t *)(ws + L.prefix);
    p.sel.sel_krem = (int *)(ws + L.krem);
    p.sel.blk_cnt = (int *)(ws + L.blk);
    p.sel.nblk = L.nblk;
    p.sel.out_idx = sel_idx; p.sel.out_val = nullptr; p.sel.out_ld = d->budget;
    p.sel.multi_ok = 1;
    p.sel.err = (int *)(ws + L.status);
    p.sel.spin_limit = g_move_spin_limit.load(std::memory_order_relaxed);
    return gather_pool_select(p, st) == hipSuccess ? REFORM_OK : REFORM_ERR_RUNTIME;
}

// ---------------------------------------------------------------------------------------
reform_status reform_embed_save_selected(const reform_embed_desc *d, const void *src, void *emb,
                                         void *hip_stream)
{
    if (!d || d->struct_size != sizeof(reform_embed_desc)) return REFORM_ERR_INVALID_ARG;
    if (d->dtype != REFORM_F32 && d->dtype != REFORM_BF16) return REFORM_ERR_INVALID_ARG;
    if (d->n_rows < 0 || d->head_dim <= 0 || d->emb_col < 0) return REFORM_ERR_INVALID_ARG;
    if (d->n_heads < 1 || (d->n_heads > 1 && d->src_head_stride < 0)) return REFORM_ERR_INVALID_ARG;
    if (d->src_row_stride < d->head_dim ||
        d->emb_row_stride < (int64_t)d->emb_col + (int64_t)d->n_heads * d->head_dim)
        return REFORM_ERR_INVALID_ARG;
    if (d->n_heads > 65535) return REFORM_ERR_UNSUPPORTED;
    if (!(d->eps > 0.f) || !std::isfinite(d->eps)) return REFORM_ERR_INVALID_ARG;
    if (d->n_rows > 0 && (!src || !emb)) return REFORM_ERR_INVALID_ARG;
    const size_t es = elt_size(d->dtype);
    const size_t row_bytes = (size_t)d->head_dim * es;
    if (row_bytes % 16 || row_bytes > 1024) return REFORM_ERR_UNSUPPORTED;
    if (((size_t)d->src_row_stride * es) % 16 || ((size_t)d->emb_row_stride * es) % 16 ||
        ((size_t)d->emb_col * es) % 16 || !aligned16(src) || !aligned16(emb))
        return REFORM_ERR_UNSUPPORTED;
    if (d->n_heads > 1 && ((size_t)d->src_head_stride * es) % 16) return REFORM_ERR_UNSUPPORTED;
    EmbedParams p;
    std::memset(&p, 0, sizeof(p));
    p.src = src; p.emb = emb; p.n_rows = d->n_rows;
    p.src_stride_bytes = (long)(d->src_row_stride * es);
    p.emb_stride_bytes = (long)(d->emb_row_stride * es);
    p.col_bytes = (long)(d->emb_col * es);
    p.n_heads = d->n_heads;
    p.src_head_bytes = d->n_heads > 1 ? (long)(d->src_head_stride * es) : 0;
    p.head_bytes = (long)row_bytes;
    p.pieces = (int)(row_bytes / 16);
    p.group = 1;
    while (p.group < p.pieces) p.group *= 2;
    p.eps = d->eps;
    return embed_save(p, d->dtype == REFORM_BF16, (hipStream_t)hip_stream) == hipSuccess
               ? REFORM_OK : REFORM_ERR_RUNTIME;
}

// ---------------------------------------------------------------------------------------
reform_status reform_rerotate_keys(const reform_rope_desc *d, void *k, const int32_t *kept_idx,
                                   void *hip_stream)
{
    if (!d || d->struct_size != sizeof(reform_rope_desc)) return REFORM_ERR_INVALID_ARG;
    if (d->dtype != REFORM_F32 && d->dtype != REFORM_BF16) return REFORM_ERR_INVALID_ARG;
    if (d->n_kv_heads <= 0 || d->head_dim <= 0 || d->capacity <= 0 || d->budget <= 0)
        return REFORM_ERR_INVALID_ARG;
    if (d->n_rows < 0 || d->n_rows > d->budget || d->n_rows > d->capacity) return REFORM_ERR_INVALID_ARG;
    if (d->rotary_dim < 0 || d->rotary_dim > d->head_dim || (d->rotary_dim % 2)) return REFORM_ERR_INVALID_ARG;
    if (!(d->theta > 1.f) || !std::isfinite(d->theta)) return REFORM_ERR_INVALID_ARG;
    if (!k || !kept_idx) return REFORM_ERR_INVALID_ARG;
    const size_t es = elt_size(d->dtype);
    if (((size_t)d->rotary_dim / 2 * es) % 16 || ((size_t)d->head_dim * es) % 16 || !aligned16(k))
        return REFORM_ERR_UNSUPPORTED;
    if (d->n_kv_heads > 65535) return REFORM_ERR_UNSUPPORTED;
    RopeParams p;
    std::memset(&p, 0, sizeof(p));
    p.k = k; p.kept = kept_idx;
    p.n_rows = d->n_rows; p.cap = d->capacity; p.kept_ld = d->budget;
    p.Hkv = d->n_kv_heads; p.rot = d->rotary_dim;
    p.row_bytes = (int)(d->head_dim * es);
    p.neg2_log2_theta_over_rot = d->rotary_dim ? -2.0 * std::log2((double)d->theta) / d->rotary_dim : 0.0;
    return rope_rerotate_launch(p, d->dtype == REFORM_BF16, (hipStream_t)hip_stream) == hipSuccess
               ? REFORM_OK : REFORM_ERR_RUNTIME;
}

// ---------------------------------------------------------------------------------------
reform_status reform_gather_rows(const reform_rows_desc *d, const void *table, const int32_t *idx,
                                 const int32_t *count, void *out, int32_t *err, void *hip_stream)
{
    if (!d || d->struct_size != sizeof(reform_rows_desc) || d->reserved != 0) return REFORM_ERR_INVALID_ARG;
    if (d->n_table <= 0 || d->n_idx < 0 || d->row_bytes <= 0) return REFORM_ERR_INVALID_ARG;
    if (!table || !out || (!idx && d->n_idx > 0)) return REFORM_ERR_INVALID_ARG;
    if (d->n_table >= (1ll << 31) || d->n_idx >= (1ll << 31)) return REFORM_ERR_UNSUPPORTED;
    if (d->row_bytes % 16 || !aligned16(table) || !aligned16(out)) return REFORM_ERR_UNSUPPORTED;
    RowsParams p;
    std::memset(&p, 0, sizeof(p));
    p.table = table; p.out = out; p.idx = idx; p.count = count; p.err = err;
    p.n_table = d->n_table; p.n_idx = d->n_idx; p.row_bytes = d->row_bytes; p.pieces = d->row_bytes / 16;
    return gather_rows_launch(p, (hipStream_t)hip_stream) == hipSuccess ? REFORM_OK : REFORM_ERR_RUNTIME;
}

// ---------------------------------------------------------------------------------------
reform_status reform_probe_mfma_bf16(const void *operands, float *sink, int32_t iters,
                                     int32_t workgroups, void *hip_stream)
{
    if (!operands || !sink || iters <= 0 || workgroups <= 0 || !aligned16(operands)) return REFORM_ERR_INVALID_ARG;
    return probe_mfma_launch(operands, sink, iters, workgroups, (hipStream_t)hip_stream) == hipSuccess
               ? REFORM_OK : REFORM_ERR_RUNTIME;
}

reform_status reform_probe_stream(const void *src, void *dst, size_t bytes, void *sink, void *hip_stream)
{
    if (!src || !sink || (bytes % 16) || !aligned16(src) || !aligned16(dst)) return REFORM_ERR_INVALID_ARG;
    return probe_stream_launch(src, dst, bytes, sink, (hipStream_t)hip_stream) == hipSuccess
               ? REFORM_OK : REFORM_ERR_RUNTIME;
}

}  // extern "C"

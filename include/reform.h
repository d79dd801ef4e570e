/*
 * reform.h -- C ABI of the MI355X (gfx950) REFORM compress-and-gather hot path.
 *
 * Three calls, named after the steps of the method (arXiv 2506.01215):
 *
 *   reform_chunk_attend_score   Alg. 1 `layer.Forward(hs, cache)`, attention part: one chunk of
 *                               queries attends causally over [compressed KV cache || chunk KV]
 *                               (Sec. 3.1, Fig. 1 step 1) and, in the same call, produces the
 *                               eviction score of every key (Sec. 3.1 compresses the cache by
 *                               evicting on attention weights, as H2O does; Sec. 5 names fusing
 *                               this score into the attention kernel as the open efficiency item).
 *   reform_evict_topk_compact   Alg. 1 `Compress(cache)`: keep the heavy hitters up to the budget
 *                               and re-pack the cache so retained tokens are consecutive
 *                               (Sec. 3.1, Sec. 1, Sec. 4 common setup).
 *   reform_gather_topk          Alg. 1 `GatherRelevant(input, emb)`: cosine similarity between
 *                               query embeddings and every context embedding, highest scores
 *                               selected, neighbourhood kept contiguous (Sec. 3.3, App. C.6).
 *
 * Conventions common to all calls
 *   - Every data pointer is a DEVICE pointer (HIP global memory) owned by the caller.  The
 *     library never allocates, frees or keeps a pointer; scratch comes in through `workspace`,
 *     whose size the matching *_workspace() query returns (bytes; 256-byte aligned base needed).
 *   - Descriptors are HOST structs; `struct_size` must be sizeof() of the struct.
 *   - Work is enqueued on `hip_stream` (a hipStream_t cast to void*; NULL = the default stream)
 *     and the call returns without synchronising.
 *   - Arguments are validated on the host before anything is launched.  On any status other
 *     than REFORM_OK nothing was launched and the outputs are unchanged, except
 *     REFORM_ERR_RUNTIME (a HIP launch failed part-way): outputs are then undefined.
 *   - No C++ type, exception or torch object crosses this boundary.
 *   - Calls on different streams may overlap if their buffers (workspace included) are disjoint.
 *   - bf16 storage is the upper 16 bits of an IEEE fp32; conversions round to nearest even.
 */
#ifndef REFORM_H
#define REFORM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    REFORM_OK = 0,
    REFORM_ERR_INVALID_ARG = 1,   /* null pointer, bad shape, wrong struct_size, ...          */
    REFORM_ERR_UNSUPPORTED = 2,   /* well-formed but outside what the kernels implement       */
    REFORM_ERR_WORKSPACE = 3,     /* workspace missing, misaligned or too small               */
    REFORM_ERR_RUNTIME = 4        /* a HIP call failed                                         */
} reform_status;

typedef enum { REFORM_F32 = 0, REFORM_BF16 = 1 } reform_dtype;

/* ------------------------------------------------------------------------------------------- */
/* reform_chunk_attend_score
 *
 * For query head h (KV head g = h / G, G = n_q_heads / n_kv_heads) and chunk row i:
 *     s_ij   = scale * <q_hi, k_gj>,  j in [0, cache_len + i]     (cache rows all visible, chunk
 *                                                                 rows causal, diagonal included)
 *     p_ij   = softmax_j(s_ij)
 *     out_hi = sum_j p_ij v_gj
 *     lse_hi = log sum_j exp(s_ij)
 *     score_gj (+)= sum_{h in group g} sum_{i >= chunk_len - W} p_ij      (attention mass key j
 *                 received from the last W = obs_window rows; Sec. 4 setup mentions W = 128 for
 *                 the H2O baseline, the chunk's whole length is the default)
 *
 * Layouts (element = dtype):
 *     q      [n_q_heads][chunk_len][head_dim]   head stride / row stride given in elements,
 *                                               head_dim contiguous, 16-byte aligned rows
 *     k, v   [n_kv_heads][capacity][head_dim]   contiguous; rows [0,cache_len) = retained cache,
 *                                               rows [cache_len, cache_len+chunk_len) = this
 *                                               chunk (the caller writes them there); rows
 *                                               beyond are never read
 *     out    like q, with its own strides, dtype as the inputs
 *     lse    [n_q_heads][chunk_len] fp32, may be NULL
 *     score  [n_kv_heads][capacity] fp32, entries [0, cache_len+chunk_len) written (added to when
 *            accumulate != 0), the rest untouched; may be NULL (attention only)
 * Arithmetic: products and sums in fp32; for bf16 the probabilities fed to the P.V product are
 * rounded to bf16, the score sums the unrounded fp32 probabilities.  Results are bitwise
 * reproducible run to run (no floating-point atomics); two cache rows holding bit-identical
 * keys receive bit-identical scores.
 * Supported: REFORM_BF16 with head_dim 64 or 128; REFORM_F32 with head_dim % 4 == 0, <= 256.
 */
typedef struct {
    uint32_t struct_size;
    int32_t  dtype;                          /* reform_dtype                                   */
    int32_t  n_q_heads, n_kv_heads, head_dim;
    int32_t  cache_len, chunk_len, capacity; /* M >= 0, C_t >= 1, capacity >= M + C_t          */
    int64_t  q_head_stride, q_row_stride;    /* elements                                       */
    int64_t  o_head_stride, o_row_stride;    /* elements                                       */
    float    scale;                          /* > 0, finite; 1/sqrt(head_dim) in the paper's models */
    int32_t  obs_window;                     /* W in [1, chunk_len]; 0 means chunk_len         */
    int32_t  accumulate;                     /* 0: score = ..., 1: score += ...                */
    int32_t  phases;                         /* 0 or 3: attention then score (the normal call);
                                                1: attention only (out, lse);
                                                2: score only, reading lse written by an earlier
                                                   phase-1 call with the same inputs (lets a
                                                   profiler bracket each kernel separately)       */
} reform_attn_desc;

size_t reform_chunk_attend_score_workspace(const reform_attn_desc *desc);

reform_status reform_chunk_attend_score(const reform_attn_desc *desc,
                                        const void *q, const void *k, const void *v,
                                        void *out, float *lse, float *score,
                                        void *workspace, size_t workspace_bytes,
                                        void *hip_stream);

/* ------------------------------------------------------------------------------------------- */
/* reform_evict_topk_compact
 *
 * Per KV head, among the n_valid = M + C_t candidate slots keep the `budget` slots with the
 * largest score (ties: the lowest slot index wins); the first n_sink and the last n_recent slots
 * are always kept and count inside the budget (Sec. 4 setup keeps the initial and recent 256
 * tokens).  Then row r of the cache becomes old row kept_idx[r] for r < new_len, in ascending
 * slot order, for k, v, score and pos alike -- in place.  new_len = min(n_valid, budget); it is
 * a function of the descriptor, nothing is read back.  If n_valid <= budget nothing moves.
 *
 *     k, v     [n_kv_heads][capacity][head_dim], in/out; rows >= new_len keep stale content
 *     score    [n_kv_heads][capacity] fp32, in/out; must be finite (no NaN/Inf)
 *     pos      [n_kv_heads][capacity] int32 token ids travelling with the rows, in/out, may be NULL
 *     kept_idx [n_kv_heads][budget] int32 out (first new_len entries per head), may be NULL
 * Supported: head_dim * sizeof(element) must be a multiple of 16; capacity <= 2^31 - 65536.
 * Device-side status: when rows move in place (row sizes that divide 16 KB), workgroups order
 * their reads and writes through flags with a bounded wait.  The wait cannot expire unless other
 * work keeps part of this call's workgroups off the device for seconds; if it does, the call
 * still ends, the cache content is then undefined, and the first int32 of the workspace, which
 * such a call clears when it starts, is set to 1.  A caller that wants to know reads that word
 * once the stream has finished.  Rows of more than 32768 candidates are selected by several
 * workgroups per row that wait for each other inside one launch (at most 128 workgroups, half of
 * what the chip holds at once); the same bounded wait and status word cover it, and more than two
 * such calls overlapping on one GPU from different streams are the one way to make it expire.
 */
typedef struct {
    uint32_t struct_size;
    int32_t  dtype;
    int32_t  n_kv_heads, head_dim;
    int32_t  n_valid, budget, capacity;
    int32_t  n_sink, n_recent;               /* n_sink + n_recent <= budget                    */
} reform_evict_desc;

size_t reform_evict_topk_compact_workspace(const reform_evict_desc *desc);

reform_status reform_evict_topk_compact(const reform_evict_desc *desc,
                                        void *k, void *v, float *score,
                                        int32_t *pos, int32_t *kept_idx,
                                        void *workspace, size_t workspace_bytes,
                                        void *hip_stream);

/* Testing aid for the device-side status word above.  Sets, for later calls in this process, how
 * many times a workgroup of the in-place move polls another workgroup's flag before it gives up
 * (default 2^22; a negative value restores the default).  0 switches publishing off as well, so
 * every wait on another workgroup expires on its first poll and the status word is set whenever
 * the kept set makes one tile depend on another: the error path can then be observed while every
 * kernel still runs to its end.  The cache content after such a call is undefined.            */
void reform_debug_set_move_spin_limit(int32_t polls);

/* reform_evict_topk_compact_static -- the same operation for callers that cannot allocate device
 * memory or carry a workspace: code running under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  It takes no workspace: the selection state, the staging rows
 * and the ordering flags live in a static device array of REFORM_STATIC_SCRATCH_BYTES that each
 * GPU the library runs on holds until the process ends.  Arguments, layouts, results and status
 * codes are those of reform_evict_topk_compact; the call allocates and frees nothing.
 *   - The device the work is meant for must be the current HIP device (the array's address on
 *     that device is looked up on the first call there).
 *   - A descriptor whose reform_evict_topk_compact_workspace() exceeds
 *     REFORM_STATIC_SCRATCH_BYTES is rejected with REFORM_ERR_WORKSPACE before any launch
 *     (8 KV heads x 65536 candidates -> 32768 of 256-byte rows needs about 5.3 MB).
 *   - Every call on a GPU shares that GPU's array, which still holds the previous call's
 *     contents; the call clears what it needs cleared itself.  Two such calls that overlap in
 *     time on one GPU (different streams or threads) race: serialise them.
 *   - The device-side status word described above is the first int32 of that array and is not
 *     reachable by the caller; use the workspace form to observe it.
 */
#define REFORM_STATIC_SCRATCH_BYTES (8u << 20)

reform_status reform_evict_topk_compact_static(const reform_evict_desc *desc,
                                               void *k, void *v, float *score,
                                               int32_t *pos, int32_t *kept_idx,
                                               void *hip_stream);

/* ------------------------------------------------------------------------------------------- */
/* reform_gather_topk
 *
 *     sim_qt   = <e_t, u_q> / max(|e_t| |u_q|, eps)              (Sec. 3.3, App. C.6)
 *     topk_q   = the k indices t with the largest sim_qt, ties to the lowest t, ascending
 *     union    = sorted unique { t + dlt : t in any topk_q, |dlt| <= radius, 0 <= t+dlt < n_ctx }
 *                united with the first n_head_keep and last n_tail_keep rows (Sec. 3.3 keeps
 *                the first and last tokens and widens hits to their neighbourhood)
 *
 *     emb         [n_ctx][dim], contiguous, dtype
 *     qry         [n_query][dim], contiguous, dtype
 *     topk_idx    [n_query][k] int32 out
 *     topk_score  [n_query][k] fp32 out (sim of the selected rows), may be NULL
 *     union_idx   [n_ctx] int32 out (first union_count entries), may be NULL (then no union)
 *     union_count one int32 in device memory, out, required iff union_idx != NULL
 * Supported: n_ctx <= 2^31 - 65536; dim % 8 == 0; any n_query >= 1 (processed 16 at a time).
 */
typedef struct {
    uint32_t struct_size;
    int32_t  dtype;
    int64_t  n_ctx;
    int32_t  dim, n_query, k;                /* 1 <= k <= n_ctx                                */
    int32_t  radius, n_head_keep, n_tail_keep;
    float    eps;                            /* > 0; 1e-8 in the tests                         */
} reform_gather_desc;

size_t reform_gather_topk_workspace(const reform_gather_desc *desc);

reform_status reform_gather_topk(const reform_gather_desc *desc,
                                 const void *emb, const void *qry,
                                 int32_t *topk_idx, float *topk_score,
                                 int32_t *union_idx, int32_t *union_count,
                                 void *workspace, size_t workspace_bytes,
                                 void *hip_stream);

/* Intermediate of reform_gather_topk, exposed for checking: only the similarity matrix,
 * sim [n_query][n_ctx] fp32 (device, out).  Same descriptor, k/radius/keeps ignored.           */
reform_status reform_gather_similarity(const reform_gather_desc *desc,
                                       const void *emb, const void *qry, float *sim,
                                       void *hip_stream);

/* ------------------------------------------------------------------------------------------- */
/* reform_gather_pooled -- the selection of Sec. 3.3 in the paper's own order
 *
 *     sim_qt   = cosine similarity as in reform_gather_topk                (Sec. 3.3, App. C.6)
 *     s_t      = max_q sim_qt                       (max-pool over the query tokens, Sec. 3.3)
 *     pooled_t = max { s_u : |u - t| <= (pool_window-1)/2, 0 <= u < n_ctx }
 *                (each token's score max-pooled with its adjacent tokens; the paper uses 128
 *                 neighbours = a window of 129, Sec. 4.5; the window is clipped at both ends)
 *     sel      = the `budget` tokens with the largest pooled_t, the first n_head_keep and the
 *                last n_tail_keep tokens always among them and counted inside the budget
 *                (Sec. 3.3 keeps the initial and final 256 tokens; Sec. 4 gives budgets of 8k and
 *                 16k), ties to the lowest index, ascending
 *
 *     emb      [n_ctx][dim], qry [n_query][dim]: contiguous, dtype
 *     sel_idx  [budget] int32 out
 *     pooled   [n_ctx] fp32 out, may be NULL (then it lives in the workspace only)
 * Supported: as reform_gather_topk; pool_window odd, 1 <= pool_window <= 1025;
 * n_head_keep + n_tail_keep <= budget <= n_ctx.
 * Device-side status: the one row of pooled scores is selected, when it has more than 32768
 * entries and at most 4 million, by up to 128 workgroups that wait for each other inside one
 * launch, with the bounded wait described for reform_evict_topk_compact; the first int32 of the
 * workspace is cleared by the call and set to 1 if such a wait expired (sel_idx is then undefined).
 */
typedef struct {
    uint32_t struct_size;
    int32_t  dtype;
    int64_t  n_ctx;
    int32_t  dim, n_query, budget;
    int32_t  pool_window, n_head_keep, n_tail_keep;
    float    eps;
} reform_pooled_desc;

size_t reform_gather_pooled_workspace(const reform_pooled_desc *desc);

reform_status reform_gather_pooled(const reform_pooled_desc *desc,
                                   const void *emb, const void *qry,
                                   int32_t *sel_idx, float *pooled,
                                   void *workspace, size_t workspace_bytes,
                                   void *hip_stream);

/* ------------------------------------------------------------------------------------------- */
/* reform_embed_save_selected -- Alg. 1 `emb.SaveSelected(qkv)`, the selected heads of one tensor
 *
 *     emb[t][col + c] = x_t[c] / max(||x_t||, eps),  c in [0, head_dim)       (Sec. 3.2, the
 *     e_comb equation: the context embedding of a token is the concatenation of the
 *     L2-normalised Q/K/V states of the selected heads; one call writes n_heads adjacent
 *     segments for the n_rows tokens of a chunk: head h is read src_head_stride elements after
 *     head h-1 and written to columns [emb_col + h*head_dim, emb_col + (h+1)*head_dim))
 *
 *     src   the first selected head's state of the chunk's first token; token t's vector starts
 *           src_row_stride elements further on for each t (so a [heads][rows][d] or a
 *           [rows][heads][d] tensor can be addressed in place); dtype
 *     emb   embedding row of the chunk's first token in the [n_ctx][emb_dim] store
 *           (emb_row_stride = emb_dim elements); dtype; only columns
 *           [emb_col, emb_col + n_heads*head_dim) of the n_rows rows are written; with
 *           n_rows = 0 nothing is read or written and both pointers may be NULL
 * Supported: head_dim * sizeof(dtype) a multiple of 16 and at most 1024 bytes; strides and
 * emb_col multiples of 16 bytes; src and emb 16-byte aligned; 1 <= n_heads <= 65535.  Sums in
 * fp32.
 */
typedef struct {
    uint32_t struct_size;
    int32_t  dtype;
    int64_t  n_rows;
    int32_t  head_dim;
    int32_t  emb_col;
    int64_t  src_row_stride, emb_row_stride; /* in elements                                    */
    float    eps;                            /* > 0; 1e-12 in the tests                        */
    int32_t  n_heads;                        /* heads written by this call (adjacent columns)  */
    int64_t  src_head_stride;                /* in elements; ignored when n_heads == 1         */
} reform_embed_desc;

reform_status reform_embed_save_selected(const reform_embed_desc *desc,
                                         const void *src, void *emb, void *hip_stream);

/* ------------------------------------------------------------------------------------------- */
/* reform_rerotate_keys -- consecutive position ids after compression (Sec. 3.1)
 *
 * For a cache that stores rotary-embedded keys: after reform_evict_topk_compact the key at slot
 * r came from slot kept_idx[r] and is rotated by delta = r - kept_idx[r] positions, in place:
 *     a           = delta * theta^(-2c/rotary_dim),              c in [0, rotary_dim/2)
 *     k'[c]       = k[c] cos a - k[c + rotary_dim/2] sin a
 *     k'[c+rd/2]  = k[c + rotary_dim/2] cos a + k[c] sin a       (half-split pairing, as in the
 *                                                               models the paper evaluates)
 * Elements [rotary_dim, head_dim) and rows with delta = 0 are not touched; V is not rotated.
 *
 *     k         [n_kv_heads][capacity][head_dim], dtype, rows [0, n_rows) rotated in place
 *     kept_idx  [n_kv_heads][budget] int32 as written by reform_evict_topk_compact
 * Angles are formed in fp64 and reduced to a fraction of a turn before the fp32 sine/cosine.
 * Supported: rotary_dim even, rotary_dim/2 * sizeof(dtype) a multiple of 16; 0 <= n_rows <=
 * min(budget, capacity).
 */
typedef struct {
    uint32_t struct_size;
    int32_t  dtype;
    int32_t  n_kv_heads, head_dim, capacity;
    int32_t  n_rows, budget;
    int32_t  rotary_dim;                     /* <= head_dim                                    */
    float    theta;                          /* rotary base, > 1 (10000, 1e6, ...)             */
} reform_rope_desc;

reform_status reform_rerotate_keys(const reform_rope_desc *desc, void *k, const int32_t *kept_idx,
                                   void *hip_stream);

/* ------------------------------------------------------------------------------------------- */
/* reform_gather_rows -- the inputs that are recomputed (Sec. 3.3 "On-Demand Cache
 * Recomputation"; Alg. 1: the selected tokens' input embeddings are gathered and forwarded again)
 *
 *     out[i] = table[idx[i]],   i in [0, n)   with n = n_idx, or min(*count, n_idx) if count != NULL
 *
 *     table  [n_table][row_bytes] bytes, any element type
 *     idx    [n_idx] int32 (the union_idx of reform_gather_topk or the sel_idx of
 *            reform_gather_pooled)
 *     count  one int32 in device memory or NULL (the union_count of reform_gather_topk, so the
 *            caller needs no host round trip)
 *     out    [n_idx][row_bytes] bytes; rows >= n are not written
 *     err    one int32 in device memory or NULL; bit 0 is set if an index was outside the
 *            table (that row is then skipped, never read); the caller clears it
 * Supported: row_bytes a multiple of 16, table and out 16-byte aligned.
 */
typedef struct {
    uint32_t struct_size;
    int32_t  reserved;                       /* 0                                              */
    int64_t  n_table, n_idx, row_bytes;
} reform_rows_desc;

reform_status reform_gather_rows(const reform_rows_desc *desc, const void *table,
                                 const int32_t *idx, const int32_t *count, void *out,
                                 int32_t *err, void *hip_stream);

/* ------------------------------------------------------------------------------------------- */
/* Measurement aids (no step of the method): what this machine sustains on the resources the
 * kernels above are bound by, so a benchmark can quote a kernel against the measured ceiling as
 * well as against the data-sheet one.
 *
 * reform_probe_mfma_bf16: `workgroups` workgroups of 8 waves each run `iters` trips of 16
 *   v_mfma_f32_16x16x32_bf16 (4 x 4 operand registers, all combinations) and nothing else;
 *   executed flop = workgroups * 8 * iters * 16 * 16384.  `operands`: 64 KiB of device memory
 *   holding the bf16 values to multiply (random data heats the chip like real inputs, zeros do
 *   not); `sink`: 16 bytes of device memory that is practically never written.
 * reform_probe_stream: reads `bytes` (a multiple of 16) from src with 16-byte loads and, if dst is
 *   not NULL, stores them to dst (a plain copy: bytes read + bytes written); with dst == NULL it
 *   is a read-only stream.  `sink` as above.
 * Both only enqueue one kernel on hip_stream.                                                   */
reform_status reform_probe_mfma_bf16(const void *operands, float *sink, int32_t iters,
                                     int32_t workgroups, void *hip_stream);
reform_status reform_probe_stream(const void *src, void *dst, size_t bytes, void *sink,
                                  void *hip_stream);

const char *reform_status_string(reform_status status);

/* Library version, major*10000 + minor*100 + patch.                                            */
int32_t reform_version(void);

#ifdef __cplusplus
}
#endif
#endif /* REFORM_H */

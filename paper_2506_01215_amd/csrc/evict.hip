// Heavy-hitter retention and order-preserving cache compaction (Sec. 3.1 of arXiv 2506.01215:
// attention-based token eviction to the budget, retained tokens re-packed to consecutive
// positions; Sec. 4 setup: protected initial / recent tokens).
//
//   select_topk    (select.hip) exact top-B of the n candidate scores per KV head, lowest-index
//                  ties, protected first/last slots, kept slot indices ascending
//   evict_move<true>   K, V rows and the score / pos entries of the kept slots -> staging
//   evict_move<false>  staging -> rows [0, new_len)
// Rows whose slot does not change (kept_idx[r] == r, always a prefix) are not touched.
#include "common.h"

namespace reform {

hipError_t select_topk(const SelParams &p, hipStream_t st);

// kept_idx = 0..n-1 when nothing is evicted (n <= B).
__global__ void evict_identity(int32_t *kept, int Hkv, int B, int n)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    const int g = blockIdx.y;
    if (r < n) kept[(size_t)g * B + r] = r;
}

// grid (ceil(B*pieces/256), Hkv, 3): z = 0 moves K rows, z = 1 V rows (one 16-byte piece per
// thread), z = 2 the 4-byte score and pos entries (one row per thread).
template <bool TO_STAGE>
__global__ __launch_bounds__(256) void evict_move(EvictParams p)
{
    const int pieces = p.row_bytes >> 4;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    const int g = blockIdx.y;
    if (blockIdx.z == 2) {
        const int r = (int)idx;
        if (idx >= p.B) return;
        const int src = p.kept[(size_t)g * p.B + r];
        if (src == r || (unsigned)src >= (unsigned)p.n) return;
        const size_t srow = (size_t)g * p.cap + (TO_STAGE ? src : r);
        const size_t trow = (size_t)g * p.B + r;
        if (TO_STAGE) {
            p.stage_score[trow] = p.score[srow];
            if (p.pos) p.stage_pos[trow] = p.pos[srow];
        } else {
            p.score[srow] = p.stage_score[trow];
            if (p.pos) p.pos[srow] = p.stage_pos[trow];
        }
        return;
    }
    const int r = (int)(idx / pieces), c = (int)(idx % pieces);
    if (r >= p.B) return;
    const int src = p.kept[(size_t)g * p.B + r];
    if (src == r || (unsigned)src >= (unsigned)p.n) return;
    const size_t srow = (size_t)g * p.cap + (TO_STAGE ? src : r);   // row in the cache arrays
    const size_t trow = (size_t)g * p.B + r;                        // row in the staging arrays
    char *cache = (char *)(blockIdx.z ? p.v : p.k) + srow * p.row_bytes + (size_t)c * 16;
    char *stage = (char *)(blockIdx.z ? p.stage_v : p.stage_k) + trow * p.row_bytes + (size_t)c * 16;
    if (TO_STAGE) *(v4u *)stage = *(const v4u *)cache;
    else *(v4u *)cache = *(const v4u *)stage;
}

hipError_t evict_run(const EvictParams &p, hipStream_t st)
{
    hipError_t e = select_topk(p.sel, st);
    if (e != hipSuccess) return e;
    const long items = (long)p.B * (p.row_bytes >> 4);
    const dim3 grid((unsigned)((items + 255) / 256), p.Hkv, 3);
    hipLaunchKernelGGL(evict_move<true>, grid, dim3(256), 0, st, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(evict_move<false>, grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

hipError_t evict_fill_identity(int32_t *kept, int Hkv, int B, int n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(evict_identity, dim3((n + 255) / 256, Hkv), dim3(256), 0, st, kept, Hkv, B, n);
    return hipGetLastError();
}

}  // namespace reform

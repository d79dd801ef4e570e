// Significance score of the gather stage as the paper states it (arXiv 2506.01215, Sec. 3.3
// "Identification of significant inputs"; window size from Sec. 4.5 "Pooling kernel size"):
// the similarities are max-pooled over the query tokens, then every context token's score is
// max-pooled with its adjacent tokens (a centred window, 129 in the paper), and the tokens with
// the highest pooled scores are selected, the first and last tokens always among them.
//
//   pool_qmax_window   one pass over sim[nq][N]: max over the nq rows while loading a tile plus
//                      its halo into LDS, then a sliding maximum by doubling (after step j every
//                      LDS slot holds the maximum of 2^j consecutive scores; a window of W is the
//                      maximum of two such spans of the largest power of two <= W), O(log W)
//                      LDS passes instead of W reads per token.
//   select_topk        (select.hip) budget selection with forced first/last slots and
//                      lowest-index ties -- pooled scores form plateaus, so ties are the rule.
#include "common.h"

namespace reform {

hipError_t select_topk(const SelParams &p, hipStream_t st);

constexpr int kPoolTile = 2048;          // context tokens per workgroup
constexpr int kPoolMaxWindow = 1025;     // odd; halo of 512 on each side
constexpr int kPoolSpan = kPoolTile + kPoolMaxWindow - 1;

__global__ __launch_bounds__(256) void pool_qmax_window(PoolParams p)
{
    __shared__ float buf[2][kPoolSpan];
    const int tid = threadIdx.x;
    const long t0 = (long)blockIdx.x * kPoolTile;
    const int h = (p.window - 1) >> 1;
    const int tile = (int)min((long)kPoolTile, p.N - t0);
    const int span = tile + p.window - 1;            // local slot i <-> token t0 - h + i
    // max over the query rows: four tokens per lane with 16-byte loads where the rows allow it,
    // the loads of several rows in flight at once (this pass reads all of sim: it is the HBM part)
    const bool quads = ((p.ld & 3) == 0) && ((h & 3) == 0) && ((((uintptr_t)p.sim) & 15) == 0);
    for (int i = 4 * tid; i < span; i += 1024) {
        const long t = t0 - h + i;
        if (quads && t >= 0 && t + 4 <= p.N && i + 4 <= span) {
            float4 m = *(const float4 *)(p.sim + t);
#pragma unroll 4
            for (int q = 1; q < p.nq; ++q) {
                const float4 v = *(const float4 *)(p.sim + (size_t)q * p.ld + t);
                m.x = fmaxf(m.x, v.x); m.y = fmaxf(m.y, v.y); m.z = fmaxf(m.z, v.z); m.w = fmaxf(m.w, v.w);
            }
            buf[0][i] = m.x; buf[0][i + 1] = m.y; buf[0][i + 2] = m.z; buf[0][i + 3] = m.w;
        } else {
            for (int j = 0; j < 4 && i + j < span; ++j) {
                const long tj = t + j;
                float m = -INFINITY;                     // outside the context: takes no part
                if (tj >= 0 && tj < p.N) {
                    m = p.sim[tj];
                    for (int q = 1; q < p.nq; ++q) m = fmaxf(m, p.sim[(size_t)q * p.ld + tj]);
                }
                buf[0][i + j] = m;
            }
        }
    }
    __syncthreads();
    int cur = 0, len = 1;
    while (2 * len <= p.window) {                    // buf[cur][i] = max of slots [i, i + len)
        for (int i = tid; i < span; i += 256) {
            const float a = buf[cur][i];
            buf[cur ^ 1][i] = i + len < span ? fmaxf(a, buf[cur][i + len]) : a;
        }
        __syncthreads();
        cur ^= 1;
        len *= 2;
    }
    // token t0 + i has the window of local slots [i, i + window)
    for (int i = tid; i < tile; i += 256)
        p.pooled[t0 + i] = fmaxf(buf[cur][i], buf[cur][i + p.window - len]);
}

hipError_t gather_pool_select(const PoolParams &p, hipStream_t st)
{
    const unsigned grid = (unsigned)((p.N + kPoolTile - 1) / kPoolTile);
    hipLaunchKernelGGL(pool_qmax_window, dim3(grid), dim3(256), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return select_topk(p.sel, st);
}

int gather_pool_max_window() { return kPoolMaxWindow; }

}  // namespace reform

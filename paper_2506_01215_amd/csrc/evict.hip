// Heavy-hitter retention and order-preserving cache compaction (Sec. 3.1 of arXiv 2506.01215:
// attention-based token eviction to the budget, retained tokens re-packed to consecutive
// positions; Sec. 4 setup: protected initial / recent tokens).
//
//   evict_select   one workgroup per KV head: exact radix select (4 x 8 bits on a monotone
//                  uint32 image of the fp32 score) of the budget-th largest key, then an ordered
//                  pass that keeps everything above the threshold plus the lowest-index ties,
//                  writes the kept slot indices ascending, and compacts score / pos in place.
//   evict_gather   K and V rows of the kept slots -> staging rows (all workgroups).
//   evict_scatter  staging rows -> rows [0, new_len) of K and V.
// Rows whose slot does not change (kept_idx[r] == r, always a prefix) are not touched.
#include "common.h"

namespace reform {


constexpr int kSelThreads = 1024;
constexpr int kSelItems = 8;     // consecutive candidates per thread per sweep of the ordered pass

// Exclusive scan of one int per thread over the workgroup; returns the exclusive prefix and the
// workgroup total.  `tmp` holds one int per wave.
__device__ __forceinline__ int block_excl_scan(int x, int *tmp, int &total)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    int incl = x;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(incl, o);
        if (lane >= o) incl += y;
    }
    __syncthreads();
    if (lane == 63) tmp[wave] = incl;
    __syncthreads();
    int base = 0, tot = 0;
    const int nw = blockDim.x >> 6;
    for (int w = 0; w < nw; ++w) {
        const int t = tmp[w];
        if (w < wave) base += t;
        tot += t;
    }
    total = tot;
    return base + incl - x;
}

__global__ __launch_bounds__(kSelThreads) void evict_select(EvictParams p)
{
    __shared__ int hist[256];
    __shared__ int suffix[257];
    __shared__ int wtmp[kSelThreads / 64];
    __shared__ uint32_t sh_prefix;
    __shared__ int sh_krem;

    const int g = blockIdx.x;
    const int tid = threadIdx.x;
    float *score = p.score + (size_t)g * p.cap;
    const int n = p.n, B = p.B;
    auto key_of = [&](int j) -> uint32_t {
        if (j < p.n_sink || j >= n - p.n_recent) return 0xffffffffu;
        return ordered_key(score[j]);
    };

    // ---- radix select of the B-th largest key, most significant byte first
    uint32_t prefix = 0;
    int krem = B;
    for (int pass = 0; pass < 4; ++pass) {
        const int shift = 24 - 8 * pass;
        if (tid < 256) hist[tid] = 0;
        __syncthreads();
        for (int j = tid; j < n; j += kSelThreads) {
            const uint32_t u = key_of(j);
            const bool match = pass == 0 || (u >> (shift + 8)) == prefix;
            if (match) atomicAdd(&hist[(u >> shift) & 255u], 1);
        }
        __syncthreads();
        // suffix[t] = number of matching keys with digit >= t
        if (tid < 256) suffix[tid] = hist[tid];
        if (tid == 0) suffix[256] = 0;
        __syncthreads();
        for (int o = 1; o < 256; o <<= 1) {
            int add = 0;
            if (tid < 256 && tid + o < 256) add = suffix[tid + o];
            __syncthreads();
            if (tid < 256) suffix[tid] += add;
            __syncthreads();
        }
        if (tid < 256 && suffix[tid + 1] < krem && krem <= suffix[tid]) {
            sh_prefix = (prefix << 8) | (uint32_t)tid;
            sh_krem = krem - suffix[tid + 1];
        }
        __syncthreads();
        prefix = sh_prefix;
        krem = sh_krem;
        __syncthreads();
    }
    const uint32_t T = prefix;    // the B-th largest key
    const int need_eq = krem;     // how many keys equal to T are kept (the lowest indices)

    // ---- ordered pass: kept slot indices, ascending
    int32_t *kept = p.kept + (size_t)g * B;
    int carry_eq = 0, carry_kept = 0;
    for (int base = 0; base < n; base += kSelThreads * kSelItems) {
        const int j0 = base + tid * kSelItems;
        uint32_t u[kSelItems];
        int eq_c = 0, gt_c = 0;
#pragma unroll
        for (int i = 0; i < kSelItems; ++i) {
            const int j = j0 + i;
            u[i] = j < n ? key_of(j) : 0u;
            const bool valid = j < n;
            gt_c += (valid && u[i] > T) ? 1 : 0;
            eq_c += (valid && u[i] == T) ? 1 : 0;
        }
        int tot_eq;
        const int eq_before = carry_eq + block_excl_scan(eq_c, wtmp, tot_eq);
        const int eq_take = max(0, min(eq_c, need_eq - eq_before));
        int tot_kept;
        int dest = carry_kept + block_excl_scan(gt_c + eq_take, wtmp, tot_kept);
        int eq_seen = eq_before;
#pragma unroll
        for (int i = 0; i < kSelItems; ++i) {
            const int j = j0 + i;
            if (j >= n) break;
            bool keep = u[i] > T;
            if (u[i] == T) {
                keep = eq_seen < need_eq;
                ++eq_seen;
            }
            if (keep && dest < B) kept[dest++] = j;
        }
        carry_eq += tot_eq;
        carry_kept += tot_kept;
    }
    __syncthreads();

    // ---- compact score and pos in place.  dest r takes slot kept[r] >= r, so sweeping dest
    // ranges in ascending order never overwrites a slot that a later range still has to read.
    int32_t *pos = p.pos ? p.pos + (size_t)g * p.cap : nullptr;
    for (int base = 0; base < B; base += kSelThreads * kSelItems) {
        float sv[kSelItems];
        int32_t pv[kSelItems];
#pragma unroll
        for (int i = 0; i < kSelItems; ++i) {
            const int r = base + i * kSelThreads + tid;
            if (r < B) {
                int src = kept[r];
                src = (unsigned)src < (unsigned)n ? src : r;
                sv[i] = score[src];
                pv[i] = pos ? pos[src] : 0;
            }
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < kSelItems; ++i) {
            const int r = base + i * kSelThreads + tid;
            if (r < B) {
                score[r] = sv[i];
                if (pos) pos[r] = pv[i];
            }
        }
        __syncthreads();
    }
}

// kept_idx = 0..n-1 when nothing is evicted (n <= B).
__global__ void evict_identity(int32_t *kept, int Hkv, int B, int n)
{
    const int r = blockIdx.x * blockDim.x + threadIdx.x;
    const int g = blockIdx.y;
    if (r < n) kept[(size_t)g * B + r] = r;
}

// grid (ceil(B*pieces/256), Hkv, 2): one 16-byte piece per thread.
__global__ __launch_bounds__(256) void evict_gather(EvictParams p)
{
    const int pieces = p.row_bytes >> 4;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    const int r = (int)(idx / pieces), c = (int)(idx % pieces);
    if (r >= p.B) return;
    const int g = blockIdx.y;
    const int src = p.kept[(size_t)g * p.B + r];
    if (src == r || (unsigned)src >= (unsigned)p.n) return;
    const char *base = (const char *)(blockIdx.z ? p.v : p.k);
    char *stage = (char *)(blockIdx.z ? p.stage_v : p.stage_k);
    const uint4 val = *(const uint4 *)(base + ((size_t)g * p.cap + src) * p.row_bytes + (size_t)c * 16);
    *(uint4 *)(stage + ((size_t)g * p.B + r) * p.row_bytes + (size_t)c * 16) = val;
}

__global__ __launch_bounds__(256) void evict_scatter(EvictParams p)
{
    const int pieces = p.row_bytes >> 4;
    const long idx = (long)blockIdx.x * 256 + threadIdx.x;
    const int r = (int)(idx / pieces), c = (int)(idx % pieces);
    if (r >= p.B) return;
    const int g = blockIdx.y;
    const int src = p.kept[(size_t)g * p.B + r];
    if (src == r || (unsigned)src >= (unsigned)p.n) return;
    char *base = (char *)(blockIdx.z ? p.v : p.k);
    const char *stage = (const char *)(blockIdx.z ? p.stage_v : p.stage_k);
    const uint4 val = *(const uint4 *)(stage + ((size_t)g * p.B + r) * p.row_bytes + (size_t)c * 16);
    *(uint4 *)(base + ((size_t)g * p.cap + r) * p.row_bytes + (size_t)c * 16) = val;
}

hipError_t evict_run(const EvictParams &p, hipStream_t st)
{
    hipLaunchKernelGGL(evict_select, dim3(p.Hkv), dim3(kSelThreads), 0, st, p);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    const long pieces = (long)p.B * (p.row_bytes >> 4);
    const dim3 grid((unsigned)((pieces + 255) / 256), p.Hkv, 2);
    hipLaunchKernelGGL(evict_gather, grid, dim3(256), 0, st, p);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(evict_scatter, grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

hipError_t evict_fill_identity(int32_t *kept, int Hkv, int B, int n, hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    hipLaunchKernelGGL(evict_identity, dim3((n + 255) / 256, Hkv), dim3(256), 0, st, kept, Hkv, B, n);
    return hipGetLastError();
}

}  // namespace reform

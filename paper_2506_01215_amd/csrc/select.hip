// Exact top-k selection per row with lowest-index ties, ascending output: the shared back end of
// the cache eviction (heavy hitters of the attention score, Sec. 3.1 of arXiv 2506.01215) and of
// the gather stage (highest similarities, Sec. 3.3).
//
//   sel_zero      clears the digit histograms (and, for a caller, a few more ints in the same launch)
//   select_hist   x3: 11 + 11 + 10 bit radix passes over the monotone uint32 image of the values;
//                 LDS histogram per workgroup of 4096 candidates, merged with integer atomics.
//                 From the second pass on every workgroup first re-derives the digit picked by
//                 the previous pass from the global histogram (8 KB of L2 reads, saves a launch).
//   select_count  final pick, then per workgroup the number of candidates above / equal to the
//                 threshold key
//   select_write  ordered emission: everything above the threshold, then the lowest-index ties
// Candidates in the first n_sink or last n_recent slots get the maximal key (always selected).
#include "common.h"

namespace reform {

constexpr int kSelBlock = 4096;      // candidates per selection workgroup (256 threads x 16)

__device__ __forceinline__ uint32_t sel_key(const SelParams &p, const float *row, long t)
{
    if (t < p.n_sink || t >= p.N - p.n_recent) return 0xffffffffu;
    return ordered_key(row[t]);
}

__device__ __forceinline__ uint32_t sel_key_of(const SelParams &p, float v, long t)
{
    if (t < p.n_sink || t >= p.N - p.n_recent) return 0xffffffffu;
    return ordered_key(v);
}

// True when the rows of `vals` can be read as aligned 16-byte quads (row pitch and base).
__device__ __forceinline__ bool sel_rows_aligned(const SelParams &p)
{
    return ((p.ld & 3) == 0) && ((((uintptr_t)p.vals) & 15) == 0);
}

__global__ void sel_zero(SelParams p)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < (long)p.nq * 3 * 2048) p.hist[i] = 0;
    if (i < p.zero_extra_n) p.zero_extra[i] = 0;
}

__device__ __forceinline__ int digit_of(uint32_t u, int pass)
{
    return pass == 0 ? (int)(u >> 21) : pass == 1 ? (int)((u >> 10) & 2047u) : (int)(u & 1023u);
}
__device__ __forceinline__ bool prefix_match(uint32_t u, uint32_t prefix, int pass)
{
    return pass == 0 ? true : pass == 1 ? (u >> 21) == prefix : (u >> 10) == prefix;
}

// Executed by all 256 threads of a workgroup: from the histogram of pass `pass` pick the digit
// that holds the k-th largest key; returns the extended prefix and the k remaining inside it.
// Every workgroup of the following kernel repeats this (8 KB of L2 reads) instead of paying a
// separate launch; workgroup 0 of each query also records the result for the kernels after it.
__device__ __forceinline__ void select_pick(const SelParams &p, int q, int pass, uint32_t &prefix,
                                            int &krem, int *part, int *sel)
{
    const int tid = threadIdx.x;
    const int *gh = p.hist + ((size_t)q * 3 + pass) * 2048;
    const uint32_t prev = pass ? p.sel_prefix[(pass - 1) * p.nq + q] : 0u;
    const int k_in = pass ? p.sel_krem[(pass - 1) * p.nq + q] : p.k;
    // thread t owns digits 8t..8t+7; suffix count of everything above its range
    int loc[8], sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { loc[i] = gh[8 * tid + i]; sum += loc[i]; }
    int total;
    const int below = block256_excl_scan(sum, part, total);   // digits of lower threads
    int acc = total - below - sum;                             // count with digit above this thread's range
#pragma unroll
    for (int i = 7; i >= 0; --i) {
        const int hi = acc;           // count with digit > 8*tid+i
        acc += loc[i];
        if (hi < k_in && k_in <= acc) { sel[0] = 8 * tid + i; sel[1] = k_in - hi; }
    }
    __syncthreads();
    const int bits = pass == 2 ? 10 : 11;
    prefix = (prev << bits) | (uint32_t)sel[0];
    krem = sel[1];
    __syncthreads();
}

// grid (nblk, nq): histogram of the current digit over the candidates matching the prefix.
__global__ __launch_bounds__(256) void select_hist(SelParams p, int pass)
{
    __shared__ int h[2048];
    __shared__ int part[256];
    __shared__ int sel[2];
    const int q = blockIdx.y, tid = threadIdx.x;
    for (int i = tid; i < 2048; i += 256) h[i] = 0;
    uint32_t prefix = 0u;
    int krem = p.k;
    if (pass) {
        select_pick(p, q, pass - 1, prefix, krem, part, sel);
        if (blockIdx.x == 0 && tid == 0) {
            p.sel_prefix[(pass - 1) * p.nq + q] = prefix;
            p.sel_krem[(pass - 1) * p.nq + q] = krem;
        }
    }
    __syncthreads();
    const float *s = p.vals + (size_t)q * p.ld;
    const long t0 = (long)blockIdx.x * kSelBlock;
    if (sel_rows_aligned(p) && t0 + kSelBlock <= p.N) {
        // full, aligned block: 16-byte loads, four candidates per lane and step
#pragma unroll
        for (int it = 0; it < kSelBlock / 1024; ++it) {
            const long t = t0 + (it * 256 + tid) * 4;
            const float4 v = *(const float4 *)(s + t);
            const float x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t u = sel_key_of(p, x[j], t + j);
                if (prefix_match(u, prefix, pass)) atomicAdd(&h[digit_of(u, pass)], 1);
            }
        }
    } else {
        for (int i = tid; i < kSelBlock; i += 256) {
            const long t = t0 + i;
            if (t < p.N) {
                const uint32_t u = sel_key(p, s, t);
                if (prefix_match(u, prefix, pass)) atomicAdd(&h[digit_of(u, pass)], 1);
            }
        }
    }
    __syncthreads();
    int *gh = p.hist + ((size_t)q * 3 + pass) * 2048;
    for (int i = tid; i < 2048; i += 256)
        if (h[i]) atomicAdd(&gh[i], h[i]);
}

// grid (nblk, nq): per block, how many candidates are above / equal to the threshold key.
__global__ __launch_bounds__(256) void select_count(SelParams p)
{
    __shared__ int red[2][4];
    __shared__ int part[256];
    __shared__ int sel[2];
    const int q = blockIdx.y, tid = threadIdx.x;
    uint32_t T;
    int need_eq;
    select_pick(p, q, 2, T, need_eq, part, sel);
    if (blockIdx.x == 0 && tid == 0) {
        p.sel_prefix[2 * p.nq + q] = T;
        p.sel_krem[2 * p.nq + q] = need_eq;
    }
    const float *s = p.vals + (size_t)q * p.ld;
    const long t0 = (long)blockIdx.x * kSelBlock;
    int gt = 0, eq = 0;
    if (sel_rows_aligned(p) && t0 + kSelBlock <= p.N) {
#pragma unroll
        for (int it = 0; it < kSelBlock / 1024; ++it) {
            const long t = t0 + (it * 256 + tid) * 4;
            const float4 v = *(const float4 *)(s + t);
            const float x[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const uint32_t u = sel_key_of(p, x[j], t + j);
                gt += u > T;
                eq += u == T;
            }
        }
    } else {
        for (int i = tid; i < kSelBlock; i += 256) {
            const long t = t0 + i;
            if (t < p.N) {
                const uint32_t u = sel_key(p, s, t);
                gt += u > T;
                eq += u == T;
            }
        }
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) { gt += __shfl_xor(gt, o); eq += __shfl_xor(eq, o); }
    if ((tid & 63) == 0) { red[0][tid >> 6] = gt; red[1][tid >> 6] = eq; }
    __syncthreads();
    if (tid == 0) {
        int *c = p.blk_cnt + ((size_t)q * p.nblk + blockIdx.x) * 2;
        c[0] = red[0][0] + red[0][1] + red[0][2] + red[0][3];
        c[1] = red[1][0] + red[1][1] + red[1][2] + red[1][3];
    }
}

// grid (nblk, nq): ordered emission of the selected indices (ascending), lowest-index ties.
__global__ __launch_bounds__(256) void select_write(SelParams p)
{
    __shared__ int tmp[4];
    __shared__ int sh_gt, sh_eq;
    const int q = blockIdx.y, tid = threadIdx.x, blk = blockIdx.x;
    const uint32_t T = p.sel_prefix[2 * p.nq + q];
    const int need_eq = p.sel_krem[2 * p.nq + q];
    // candidates above / equal to T in the blocks before this one
    const int *c = p.blk_cnt + (size_t)q * p.nblk * 2;
    int gt_b = 0, eq_b = 0;
    for (int b = tid; b < blk; b += 256) { gt_b += c[2 * b]; eq_b += c[2 * b + 1]; }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) { gt_b += __shfl_xor(gt_b, o); eq_b += __shfl_xor(eq_b, o); }
    if (tid == 0) { sh_gt = 0; sh_eq = 0; }
    __syncthreads();
    if ((tid & 63) == 0) { atomicAdd(&sh_gt, gt_b); atomicAdd(&sh_eq, eq_b); }
    __syncthreads();
    const int base_gt = sh_gt, base_eq = sh_eq;

    const float *s = p.vals + (size_t)q * p.ld;
    const long t0 = (long)blk * kSelBlock + tid * 16;
    uint32_t u[16];
    float val[16];
    int gt_c = 0, eq_c = 0;
    if (sel_rows_aligned(p) && t0 + 16 <= p.N) {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const float4 v = *(const float4 *)(s + t0 + 4 * j);
            val[4 * j] = v.x; val[4 * j + 1] = v.y; val[4 * j + 2] = v.z; val[4 * j + 3] = v.w;
        }
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            u[i] = sel_key_of(p, val[i], t0 + i);
            gt_c += u[i] > T;
            eq_c += u[i] == T;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) {
            const long t = t0 + i;
            const bool valid = t < p.N;
            val[i] = valid ? s[t] : 0.f;
            u[i] = valid ? sel_key(p, s, t) : 0u;
            gt_c += valid && u[i] > T;
            eq_c += valid && u[i] == T;
        }
    }
    int tot;
    const int eq_before = base_eq + block256_excl_scan(eq_c, tmp, tot);
    const int eq_take = max(0, min(eq_c, need_eq - eq_before));
    const int kept_before_blk = base_gt + min(base_eq, need_eq);
    int dest = kept_before_blk + block256_excl_scan(gt_c + eq_take, tmp, tot);
    int eq_seen = eq_before;
    int32_t *orank = p.out_rank ? p.out_rank + (size_t)q * p.ld : nullptr;
    int32_t *oi = p.out_idx + (size_t)q * p.out_ld;
    float *os = p.out_val ? p.out_val + (size_t)q * p.out_ld : nullptr;
    const int32_t *ss = p.side_src ? p.side_src + (size_t)q * p.ld : nullptr;
    int32_t *sd = p.side_src ? p.side_dst + (size_t)q * p.out_ld : nullptr;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const long t = t0 + i;
        if (t >= p.N) break;
        if (orank) orank[t] = dest;
        bool keep = u[i] > T;
        if (u[i] == T) { keep = eq_seen < need_eq; ++eq_seen; }
        if (keep && dest < p.k) {
            oi[dest] = (int32_t)t;
            if (os) os[dest] = val[i];
            if (ss) sd[dest] = ss[t];
            ++dest;
        }
    }
}


#define RF_CHECK_LAUNCH()                     \
    do {                                      \
        hipError_t e_ = hipGetLastError();    \
        if (e_ != hipSuccess) return e_;      \
    } while (0)

hipError_t select_topk(const SelParams &p, hipStream_t st)
{
    const long nz = max((long)p.nq * 3 * 2048, (long)p.zero_extra_n);
    hipLaunchKernelGGL(sel_zero, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, st, p);
    RF_CHECK_LAUNCH();
    const dim3 sgrid(p.nblk, p.nq);
    for (int pass = 0; pass < 3; ++pass) {
        hipLaunchKernelGGL(select_hist, sgrid, dim3(256), 0, st, p, pass);
        RF_CHECK_LAUNCH();
    }
    hipLaunchKernelGGL(select_count, sgrid, dim3(256), 0, st, p);
    RF_CHECK_LAUNCH();
    hipLaunchKernelGGL(select_write, sgrid, dim3(256), 0, st, p);
    RF_CHECK_LAUNCH();
    return hipSuccess;
}

}  // namespace reform

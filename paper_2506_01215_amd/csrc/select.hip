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
//   select_fused  rows of at most 32768 candidates: all of the above in one launch, one workgroup
//                 per row, keys held in registers
//   select_multi  longer rows, when every workgroup of the launch fits on the chip at once: one
//                 launch, several workgroups per row that wait for each other (keys in registers)
// Candidates in the first n_sink or last n_recent slots get the maximal key (always selected).
#include "common.h"

#include <atomic>

namespace reform {

constexpr int kSelBlock = 4096;      // candidates per selection workgroup (256 threads x 16)
constexpr int kHistWorkgroups = 2048; // the histogram passes use about this many workgroups at most

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
    if (p.multi_ok && i < (long)p.nq * p.nblk * 2) p.blk_cnt[i] = 0;
    if (p.err && i == 0) *p.err = 0;
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

// grid (<= nblk, nq): histogram of the current digit over the candidates matching the prefix.
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
    // a workgroup takes every gridDim.x-th block of 4096 candidates (long rows: fewer, longer
    // workgroups, so the pick above and the merge below are paid less often)
    for (int blk = blockIdx.x; blk < p.nblk; blk += gridDim.x) {
        const long t0 = (long)blk * kSelBlock;
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

// ------------------------------------------------------------------------------------------
// Building blocks shared by the ordered emission of the multi-launch path and by the
// single-launch selection of short rows.  A wave owns a contiguous range of NIT * 256
// candidates starting at w_lo; in step `it` lane l holds the four consecutive candidates
// w_lo + it * 256 + 4 * l + (0..3).  Every global access of a step is then one contiguous block
// per wave, and positions in index order follow from wave ballots (no cross-lane data movement)
// plus the running counts of the wave.  `FULL` marks a wave whose whole range lies inside the row
// (no per-candidate bounds test).
__device__ __forceinline__ int lanes_below(unsigned long long m)
{
    return (int)__builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
}

// Keys of the wave's range; slots at or beyond N hold 0 and are masked by the users.
template <int NIT>
__device__ __forceinline__ void range_keys(const SelParams &p, const float *s, int N, int w_lo, uint32_t (&u)[NIT][4])
{
    const int t_lane = w_lo + (threadIdx.x & 63) * 4;
    const int w_hi = w_lo + NIT * 256;
    const bool forced = w_lo < p.n_sink || w_hi > N - p.n_recent;     // some slot of the range may be forced in
    if (w_hi <= N && !forced && sel_rows_aligned(p)) {
#pragma unroll
        for (int it = 0; it < NIT; ++it) {
            const float4 v = *(const float4 *)(s + t_lane + it * 256);
            u[it][0] = ordered_key(v.x);
            u[it][1] = ordered_key(v.y);
            u[it][2] = ordered_key(v.z);
            u[it][3] = ordered_key(v.w);
        }
    } else {
#pragma unroll
        for (int it = 0; it < NIT; ++it)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int t = t_lane + it * 256 + j;
                const uint32_t key = sel_key(p, s, min(t, N - 1));
                u[it][j] = t < N ? key : 0u;
            }
    }
}

// Candidates of the wave's range above / equal to the threshold key (wave-uniform results).
template <int NIT, bool FULL>
__device__ __forceinline__ void range_count(const uint32_t (&u)[NIT][4], int N, int w_lo, uint32_t T, int &gt, int &eq)
{
    const int t_lane = w_lo + (threadIdx.x & 63) * 4;
    gt = 0;
    eq = 0;
#pragma unroll
    for (int it = 0; it < NIT; ++it)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const bool valid = FULL || t_lane + it * 256 + j < N;
            gt += __popcll(__ballot(valid && u[it][j] > T));
            eq += __popcll(__ballot(valid && u[it][j] == T));
        }
}

// Four consecutive 4-byte entries src[t..t+3] (those at or beyond N come back as 0).
template <bool FULL>
__device__ __forceinline__ int4 load_quad(const int32_t *src, bool quads, int t, int N)
{
    if (quads && (FULL || t + 4 <= N)) return *(const int4 *)(src + t);
    int4 r;
    r.x = t < N ? src[t] : 0;
    r.y = t + 1 < N ? src[t + 1] : 0;
    r.z = t + 2 < N ? src[t + 2] : 0;
    r.w = t + 3 < N ? src[t + 3] : 0;
    return r;
}

// Ordered emission of the wave's range: dest_run = selected candidates before the range,
// eq_run = candidates equal to T before it (both wave-uniform).  The values and the companion
// entries of a step are fetched as whole quads one step ahead, never per selected candidate
// (a load feeding a store inside the per-candidate branch costs a memory round trip each).
template <int NIT, bool FULL>
__device__ __forceinline__ void range_emit(const SelParams &p, int q, const uint32_t (&u)[NIT][4], int N, int w_lo,
                                           uint32_t T, int need_eq, int dest_run, int eq_run)
{
    const int t_lane = w_lo + (threadIdx.x & 63) * 4;
    const int32_t *sv = (const int32_t *)(p.vals + (size_t)q * p.ld);
    int32_t *orank = p.out_rank ? p.out_rank + (size_t)q * p.ld : nullptr;
    const bool rank_quads = ((p.ld & 3) == 0) && ((((uintptr_t)p.out_rank) & 15) == 0);
    const bool val_quads = sel_rows_aligned(p);
    const bool side_quads = ((p.ld & 3) == 0) && ((((uintptr_t)p.side_src) & 15) == 0);
    int32_t *oi = p.out_idx + (size_t)q * p.out_ld;
    int32_t *os = p.out_val ? (int32_t *)(p.out_val + (size_t)q * p.out_ld) : nullptr;
    const int32_t *ss = p.side_src ? p.side_src + (size_t)q * p.ld : nullptr;
    int32_t *sd = p.side_src ? p.side_dst + (size_t)q * p.out_ld : nullptr;
    int4 val_nx = make_int4(0, 0, 0, 0), side_nx = make_int4(0, 0, 0, 0);
    if (os) val_nx = load_quad<FULL>(sv, val_quads, t_lane, N);
    if (ss) side_nx = load_quad<FULL>(ss, side_quads, t_lane, N);
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int t = t_lane + it * 256;
        const int4 val4 = val_nx, side4 = side_nx;
        if (it + 1 < NIT) {
            if (os) val_nx = load_quad<FULL>(sv, val_quads, t + 256, N);
            if (ss) side_nx = load_quad<FULL>(ss, side_quads, t + 256, N);
        }
        const int val[4] = {val4.x, val4.y, val4.z, val4.w};
        const int side[4] = {side4.x, side4.y, side4.z, side4.w};
        bool keep[4];
        unsigned long long me[4];
        unsigned long long any_eq = 0;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            me[j] = __ballot((FULL || t + j < N) && u[it][j] == T);
            any_eq |= me[j];
        }
        if (any_eq) {                                         // ties inside these 256 candidates: lowest index first
            int eq_seen = eq_run;
#pragma unroll
            for (int j = 0; j < 4; ++j) eq_seen += lanes_below(me[j]);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const bool is_eq = (FULL || t + j < N) && u[it][j] == T;
                keep[j] = (FULL || t + j < N) && (u[it][j] > T || (is_eq && eq_seen < need_eq));
                eq_seen += is_eq;
                eq_run += __popcll(me[j]);
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) keep[j] = (FULL || t + j < N) && u[it][j] > T;
        }
        int dest = dest_run;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const unsigned long long mk = __ballot(keep[j]);
            dest += lanes_below(mk);
            dest_run += __popcll(mk);
        }
        if (orank) {
            const int r1 = dest + keep[0], r2 = r1 + keep[1], r3 = r2 + keep[2];
            if (rank_quads && (FULL || t + 4 <= N)) {
                *(int4 *)(orank + t) = make_int4(dest, r1, r2, r3);
            } else {
                if (t < N) orank[t] = dest;
                if (t + 1 < N) orank[t + 1] = r1;
                if (t + 2 < N) orank[t + 2] = r2;
                if (t + 3 < N) orank[t + 3] = r3;
            }
        }
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (keep[j] && (unsigned)dest < (unsigned)p.k) {
                oi[dest] = (int32_t)(t + j);
                if (os) os[dest] = val[j];
                if (ss) sd[dest] = side[j];
            }
            dest += keep[j];
        }
    }
}

// grid (nblk, nq): ordered emission of the selected indices (ascending), lowest-index ties.
// A workgroup covers 4096 candidates, a wave 1024 of them.
__global__ __launch_bounds__(256) void select_write(SelParams p)
{
    __shared__ int wtot[2][4];
    __shared__ int sh_gt, sh_eq;
    const int q = blockIdx.y, tid = threadIdx.x, blk = blockIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
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
    if (lane == 0) { atomicAdd(&sh_gt, gt_b); atomicAdd(&sh_eq, eq_b); }

    const float *s = p.vals + (size_t)q * p.ld;
    const int N = (int)p.N;
    const int w_lo = blk * kSelBlock + wave * 1024;
    const bool full = w_lo + 1024 <= N;
    uint32_t u[4][4];
    range_keys<4>(p, s, N, w_lo, u);
    int gt_w, eq_w;
    if (full) range_count<4, true>(u, N, w_lo, T, gt_w, eq_w);
    else range_count<4, false>(u, N, w_lo, T, gt_w, eq_w);
    if (lane == 0) { wtot[0][wave] = gt_w; wtot[1][wave] = eq_w; }
    __syncthreads();
    int base_gt = sh_gt, base_eq = sh_eq;                         // above / equal to T before this wave's range
#pragma unroll
    for (int w = 0; w < 4; ++w)
        if (w < wave) { base_gt += wtot[0][w]; base_eq += wtot[1][w]; }
    const int dest_run = base_gt + min(base_eq, need_eq);
    if (full) range_emit<4, true>(p, q, u, N, w_lo, T, need_eq, dest_run, base_eq);
    else range_emit<4, false>(p, q, u, N, w_lo, T, need_eq, dest_run, base_eq);
}

// ------------------------------------------------------------------------------------------
// Rows of at most 32768 candidates: the whole selection of a row in ONE launch by one workgroup
// of 1024 threads (16 waves, each owning NIT * 256 candidates).  The row is read once; its keys
// stay in registers through the three radix passes (LDS histogram, pick by a workgroup scan) and
// the ordered emission.  Results are identical to the multi-launch path; the per-pass selection
// state is not written back.  One compute unit does all the work of a row, so beyond this size
// the multi-launch path, which spreads a row over many, is faster.
constexpr int kFusedMaxN = 32768;

// Histogram of digit PASS over the keys a thread holds (candidates matching the prefix only).
template <int NIT, int PASS, bool FULL>
__device__ __forceinline__ void fused_hist(const uint32_t (&u)[NIT][4], int N, int w_lo, uint32_t prefix, int *h)
{
    const int lane = threadIdx.x & 63;
    const int t_lane = w_lo + lane * 4;
#pragma unroll
    for (int it = 0; it < NIT; ++it) {
        const int t = t_lane + it * 256;
        bool m[4];
        bool same = true;                                     // all four count and share one digit
        const int d0 = digit_of(u[it][0], PASS);
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            m[j] = (FULL || t + j < N) && prefix_match(u[it][j], prefix, PASS);
            same = same && m[j] && digit_of(u[it][j], PASS) == d0;
        }
        // a wave whose 256 candidates all fall into one bin adds them at once (constant or
        // narrowly spread rows would otherwise serialise 64 lanes on one LDS address)
        const int dref = __builtin_amdgcn_readfirstlane(d0);
        if (__all(same && d0 == dref)) {
            if (lane == 0) atomicAdd(&h[dref], 256);
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (m[j]) atomicAdd(&h[digit_of(u[it][j], PASS)], 1);
        }
    }
}

// Executed by all 1024 threads: pick the digit of the histogram that holds the krem-th largest
// key (thread t owns digits 2t and 2t+1) and extend the prefix by it.
template <int PASS>
__device__ __forceinline__ void fused_pick(uint32_t &prefix, int &krem, const int *h, int *wtot, int *sel)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l0 = h[2 * tid], l1 = h[2 * tid + 1], sum = l0 + l1;
    int incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(incl, o);
        if (lane >= o) incl += y;
    }
    if (lane == 63) wtot[wave] = incl;
    __syncthreads();
    int below = incl - sum, total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const int x = wtot[w];
        if (w < wave) below += x;
        total += x;
    }
    const int above = total - below - sum;                    // candidates with a digit above 2t+1
    if (above < krem && krem <= above + l1) { sel[0] = 2 * tid + 1; sel[1] = krem - above; }
    else if (above + l1 < krem && krem <= above + sum) { sel[0] = 2 * tid; sel[1] = krem - above - l1; }
    __syncthreads();
    prefix = (prefix << (PASS == 2 ? 10 : 11)) | (uint32_t)sel[0];
    krem = sel[1];
    __syncthreads();
}

template <int NIT>
__global__ __launch_bounds__(1024) void select_fused(SelParams p)
{
    __shared__ int h[2048];
    __shared__ int wtot[2][16];
    __shared__ int sel[2];
    const int q = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    for (long i = (long)q * 1024 + tid; i < p.zero_extra_n; i += (long)gridDim.x * 1024) p.zero_extra[i] = 0;

    const float *s = p.vals + (size_t)q * p.ld;
    const int N = (int)p.N;
    const int w_lo = wave * (NIT * 256);
    const bool full = w_lo + NIT * 256 <= N;
    uint32_t u[NIT][4];
    range_keys<NIT>(p, s, N, w_lo, u);

    uint32_t prefix = 0u;
    int krem = p.k;
#define RF_FUSED_PASS(PASS)                                                           \
    for (int i = tid; i < 2048; i += 1024) h[i] = 0;                                  \
    __syncthreads();                                                                  \
    if (full) fused_hist<NIT, PASS, true>(u, N, w_lo, prefix, h);                     \
    else fused_hist<NIT, PASS, false>(u, N, w_lo, prefix, h);                         \
    __syncthreads();                                                                  \
    fused_pick<PASS>(prefix, krem, h, wtot[0], sel);
    RF_FUSED_PASS(0)
    RF_FUSED_PASS(1)
    RF_FUSED_PASS(2)
#undef RF_FUSED_PASS
    const uint32_t T = prefix;                                    // key of the k-th largest candidate
    const int need_eq = krem;                                     // how many candidates equal to it are taken

    int gt_w, eq_w;
    if (full) range_count<NIT, true>(u, N, w_lo, T, gt_w, eq_w);
    else range_count<NIT, false>(u, N, w_lo, T, gt_w, eq_w);
    if (lane == 0) { wtot[0][wave] = gt_w; wtot[1][wave] = eq_w; }
    __syncthreads();
    int base_gt = 0, base_eq = 0;                                 // above / equal to T in the waves before this one
#pragma unroll
    for (int w = 0; w < 16; ++w)
        if (w < wave) { base_gt += wtot[0][w]; base_eq += wtot[1][w]; }
    const int dest_run = base_gt + min(base_eq, need_eq);
    if (full) range_emit<NIT, true>(p, q, u, N, w_lo, T, need_eq, dest_run, base_eq);
    else range_emit<NIT, false>(p, q, u, N, w_lo, T, need_eq, dest_run, base_eq);
}

// ------------------------------------------------------------------------------------------
// Rows longer than that, in ONE launch when the whole grid can be resident at once: `parts`
// workgroups of 1024 threads share a row, each holding NIT * 4096 of its candidates in registers
// for the whole selection.  Per radix pass a workgroup merges its LDS histogram into the row's
// global histogram (cleared by the launch before) with integer atomics and then polls that
// histogram until its total equals the number of candidates the pass must see -- all N in the
// first pass, afterwards the count of the bin picked by the pass before -- so the merged histogram
// is its own completion signal and no separate barrier is paid.  Every workgroup of a row takes
// the same pick from the same numbers.  The per-workgroup counts of candidates above / equal to
// the threshold are published as count + 1 into cleared words, which the later workgroups of the
// row poll for; from them each workgroup derives where its share of the ascending output starts.
// Results are identical to the other two paths.
//
// Everything that crosses workgroups inside the launch goes through agent-scope atomics (adds,
// loads, stores), which are performed beyond the per-XCD L2s.  The waits are bounded: the host
// launches this kernel only with at most kMultiMaxGroups workgroups, half of what the chip's 256
// compute units hold at once even at one such workgroup each, so every workgroup that is waited
// for is running or will be dispatched as soon as unrelated work drains; if a limit is reached
// all the same (more than two such launches overlapping on different streams could do that), the
// kernel still ends, sets *err and leaves undefined output.
constexpr int kMultiMaxGroups = 128;

// All 1024 threads: poll the row's histogram of a pass (thread t owns digits 2t, 2t+1) until it
// holds `expected` candidates, then leave that snapshot in h.
__device__ __forceinline__ void multi_wait_hist(const int *gh, int ndigits, int expected, int *h, int *wtot,
                                                int spin_limit, int *err)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    int v0 = 0, v1 = 0;
    for (int spins = 0;; ++spins) {
        if (2 * tid < ndigits) {
            v0 = __hip_atomic_load(&gh[2 * tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            v1 = __hip_atomic_load(&gh[2 * tid + 1], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        }
        int sum = v0 + v1;
#pragma unroll
        for (int o = 32; o >= 1; o >>= 1) sum += __shfl_xor(sum, o);
        if (lane == 0) wtot[wave] = sum;
        __syncthreads();
        int total = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) total += wtot[w];
        __syncthreads();                                  // wtot is rewritten by the next poll
        if (total == expected) break;
        if (spins >= spin_limit) {                        // uniform: every thread saw the same total
            if (tid == 0 && err) atomicExch(err, 1);
            break;
        }
        __builtin_amdgcn_s_sleep(1);
    }
    h[2 * tid] = v0;
    h[2 * tid + 1] = v1;
    __syncthreads();
}

// fused_pick that also reports how many candidates the picked digit holds (sel[2]).
template <int PASS>
__device__ __forceinline__ void multi_pick(uint32_t &prefix, int &krem, int &in_bin, const int *h, int *wtot, int *sel)
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l0 = h[2 * tid], l1 = h[2 * tid + 1], sum = l0 + l1;
    int incl = sum;
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int y = __shfl_up(incl, o);
        if (lane >= o) incl += y;
    }
    if (lane == 63) wtot[wave] = incl;
    __syncthreads();
    int below = incl - sum, total = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) {
        const int x = wtot[w];
        if (w < wave) below += x;
        total += x;
    }
    const int above = total - below - sum;                    // candidates with a digit above 2t+1
    if (above < krem && krem <= above + l1) { sel[0] = 2 * tid + 1; sel[1] = krem - above; sel[2] = l1; }
    else if (above + l1 < krem && krem <= above + sum) { sel[0] = 2 * tid; sel[1] = krem - above - l1; sel[2] = l0; }
    __syncthreads();
    prefix = (prefix << (PASS == 2 ? 10 : 11)) | (uint32_t)sel[0];
    krem = sel[1];
    in_bin = sel[2];
    __syncthreads();
}

template <int NIT>
__global__ __launch_bounds__(1024) void select_multi(SelParams p, int parts)
{
    __shared__ int h[2048];
    __shared__ int wtot[2][16];
    __shared__ int sel[3];
    __shared__ int before[2];
    const int q = blockIdx.x / parts, part = blockIdx.x % parts;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid < 3) sel[tid] = 0;
    if (tid < 2) before[tid] = 0;

    const float *s = p.vals + (size_t)q * p.ld;
    const int N = (int)p.N;
    const int w_lo = part * (NIT * 4096) + wave * (NIT * 256);
    const bool full = w_lo + NIT * 256 <= N;
    uint32_t u[NIT][4];
    range_keys<NIT>(p, s, N, w_lo, u);

    uint32_t prefix = 0u;
    int krem = p.k;
    int expected = N;                                             // candidates the coming pass counts
#define RF_MULTI_PASS(PASS)                                                                  \
    {                                                                                        \
        for (int i = tid; i < 2048; i += 1024) h[i] = 0;                                     \
        __syncthreads();                                                                     \
        if (full) fused_hist<NIT, PASS, true>(u, N, w_lo, prefix, h);                        \
        else fused_hist<NIT, PASS, false>(u, N, w_lo, prefix, h);                            \
        __syncthreads();                                                                     \
        int *gh = p.hist + ((size_t)q * 3 + PASS) * 2048;                                    \
        for (int i = tid; i < 2048; i += 1024)                                               \
            if (h[i]) atomicAdd(&gh[i], h[i]);                                               \
        __syncthreads();                                                                     \
        multi_wait_hist(gh, PASS == 2 ? 1024 : 2048, expected, h, wtot[0], p.spin_limit, p.err); \
        multi_pick<PASS>(prefix, krem, expected, h, wtot[0], sel);                           \
    }
    RF_MULTI_PASS(0)
    RF_MULTI_PASS(1)
    RF_MULTI_PASS(2)
#undef RF_MULTI_PASS
    const uint32_t T = prefix;
    const int need_eq = max(krem, 0);

    int gt_w, eq_w;
    if (full) range_count<NIT, true>(u, N, w_lo, T, gt_w, eq_w);
    else range_count<NIT, false>(u, N, w_lo, T, gt_w, eq_w);
    if (lane == 0) { wtot[0][wave] = gt_w; wtot[1][wave] = eq_w; }
    __syncthreads();
    int *c = p.blk_cnt + (size_t)q * parts * 2;                   // cleared words: 0 = not published yet
    if (tid < 2) {
        int tot = 0;
#pragma unroll
        for (int w = 0; w < 16; ++w) tot += wtot[tid][w];
        __hip_atomic_store(&c[2 * part + tid], tot + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // candidates above / equal to T in the workgroups before this one (2 * parts <= 256 < 1024 threads)
    if (tid < 2 * part) {
        int v = 0;
        for (int spins = 0;; ++spins) {
            v = __hip_atomic_load(&c[tid], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if (v != 0) break;
            if (spins >= p.spin_limit) {
                if (p.err) atomicExch(p.err, 1);
                v = 1;
                break;
            }
            __builtin_amdgcn_s_sleep(1);
        }
        atomicAdd(&before[tid & 1], v - 1);
    }
    __syncthreads();
    int base_gt = before[0], base_eq = before[1];
#pragma unroll
    for (int w = 0; w < 16; ++w)
        if (w < wave) { base_gt += wtot[0][w]; base_eq += wtot[1][w]; }
    const int dest_run = base_gt + min(base_eq, need_eq);
    if (full) range_emit<NIT, true>(p, q, u, N, w_lo, T, need_eq, dest_run, base_eq);
    else range_emit<NIT, false>(p, q, u, N, w_lo, T, need_eq, dest_run, base_eq);
}

#define RF_CHECK_LAUNCH()                     \
    do {                                      \
        hipError_t e_ = hipGetLastError();    \
        if (e_ != hipSuccess) return e_;      \
    } while (0)

// Compute units of the current device (cached per device; 256 on an unpartitioned MI355X).
static int device_compute_units()
{
    static std::atomic<int> cached[64];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
    int v = cached[dev].load(std::memory_order_relaxed);
    if (v > 0) return v;
    if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || v <= 0) return 0;
    cached[dev].store(v, std::memory_order_relaxed);
    return v;
}

hipError_t select_topk(const SelParams &p, hipStream_t st)
{
    if (p.N <= kFusedMaxN) {
        if (p.N <= 4096) hipLaunchKernelGGL(select_fused<1>, dim3(p.nq), dim3(1024), 0, st, p);
        else if (p.N <= 8192) hipLaunchKernelGGL(select_fused<2>, dim3(p.nq), dim3(1024), 0, st, p);
        else if (p.N <= 16384) hipLaunchKernelGGL(select_fused<4>, dim3(p.nq), dim3(1024), 0, st, p);
        else hipLaunchKernelGGL(select_fused<8>, dim3(p.nq), dim3(1024), 0, st, p);
        RF_CHECK_LAUNCH();
        return hipSuccess;
    }
    if (!p.pre_zeroed) {
        const long nz = max((long)p.nq * 3 * 2048, (long)p.zero_extra_n);
        hipLaunchKernelGGL(sel_zero, dim3((unsigned)((nz + 255) / 256)), dim3(256), 0, st, p);
        RF_CHECK_LAUNCH();
    }
    // one launch for the rest when the row's workgroups can all be resident together
    if (p.multi_ok) {
        // at most half of the compute units (a partitioned device has fewer than 256)
        const long max_groups = min((long)kMultiMaxGroups, (long)device_compute_units() / 2);
        for (int nit = 1; nit <= 8; nit *= 2) {
            const long parts = (p.N + (long)nit * 4096 - 1) / ((long)nit * 4096);
            if ((long)p.nq * parts > max_groups) continue;
            const dim3 grid((unsigned)(p.nq * parts));
            if (nit == 1) hipLaunchKernelGGL(select_multi<1>, grid, dim3(1024), 0, st, p, (int)parts);
            else if (nit == 2) hipLaunchKernelGGL(select_multi<2>, grid, dim3(1024), 0, st, p, (int)parts);
            else if (nit == 4) hipLaunchKernelGGL(select_multi<4>, grid, dim3(1024), 0, st, p, (int)parts);
            else hipLaunchKernelGGL(select_multi<8>, grid, dim3(1024), 0, st, p, (int)parts);
            RF_CHECK_LAUNCH();
            return hipSuccess;
        }
    }
    const dim3 sgrid(p.nblk, p.nq);
    const int hblk = max(1, kHistWorkgroups / p.nq);       // workgroups per row of the histogram passes
    const dim3 hgrid(min(p.nblk, hblk), p.nq);
    for (int pass = 0; pass < 3; ++pass) {
        hipLaunchKernelGGL(select_hist, hgrid, dim3(256), 0, st, p, pass);
        RF_CHECK_LAUNCH();
    }
    hipLaunchKernelGGL(select_count, sgrid, dim3(256), 0, st, p);
    RF_CHECK_LAUNCH();
    hipLaunchKernelGGL(select_write, sgrid, dim3(256), 0, st, p);
    RF_CHECK_LAUNCH();
    return hipSuccess;
}

}  // namespace reform

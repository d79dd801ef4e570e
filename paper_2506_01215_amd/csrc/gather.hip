// Gather stage (Sec. 3.3 "Identification of significant inputs" and App. C.6 "Similarity search"
// of arXiv 2506.01215): cosine similarity of query embeddings with every context embedding,
// per-query top-k with lowest-index ties, union with a +-radius neighbourhood, sorted unique.
//
//   sim_bf16_mfma   streams the [N][D] bf16 store once; 16 rows x up to 16 queries per
//                   v_mfma_f32_16x16x32_bf16; the row norms come from a second MFMA of the row
//                   tile with itself (Gram diagonal), so the VALU does no per-element work and
//                   the kernel stays HBM-bound for 16 queries.
//   sim_generic     fp32 (or odd-shaped bf16) inputs: one wave per row, fp32 FMA.
//   select_*        3-pass radix select (11+11+10 bits) of the k-th largest per query with
//                   histograms in LDS, then an ordered two-kernel compaction.
//   union_*         bitmap of N bits: mark dilated hits, count, emit ascending.
#include "common.h"

namespace reform {


constexpr int kSelBlock = 4096;      // candidates per selection workgroup (256 threads x 16)
constexpr int kUnionWordsPerBlock = 1024;

// ------------------------------------------------------------------------------------------
// 16x16x32 operand layout (wave64): A[m][k]: lane l holds m = l%16, k = 8*(l/16)..+7;
// B[k][n]: lane l holds n = l%16, same k;  C[m][n]: lane l holds n = l%16, m = 4*(l/16) + e.
__global__ __launch_bounds__(256) void sim_bf16_mfma(GatherParams p)
{
    extern __shared__ __attribute__((aligned(16))) u16 qs[];   // [16][D+8]
    __shared__ float qnorm[16];
    const int D = p.D, QROW = D + 8;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, lg = lane >> 4;

    // stage the (up to 16) queries of this group, zero-padded, and their norms
    const u16 *Q = (const u16 *)p.qry + (size_t)p.q0 * D;
    for (int idx = tid; idx < 16 * (D / 8); idx += 256) {
        const int r = idx / (D / 8), c8 = idx % (D / 8);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (r < p.nq_grp) v = *(const uint4 *)(Q + (size_t)r * D + c8 * 8);
        *(uint4 *)(qs + r * QROW + c8 * 8) = v;
    }
    __syncthreads();
    if (wave == 0) {
        // 4 lanes per query, fixed order
        float s = 0.f;
        for (int c = lg; c < D; c += 4) {
            const float x = bf16_bits_to_f32(qs[ln * QROW + c]);
            s = fmaf(x, x, s);
        }
        s += __shfl_xor(s, 16);
        s += __shfl_xor(s, 32);
        if (lg == 0) qnorm[ln] = sqrtf(s);
    }
    __syncthreads();
    const float un = qnorm[ln];

    const long ngroups = (p.N + 15) / 16;
    const long stride = (long)gridDim.x * 4;
    const u16 *E = (const u16 *)p.emb;
    for (long grp = (long)blockIdx.x * 4 + wave; grp < ngroups; grp += stride) {
        const long row0 = grp * 16;
        long row = row0 + ln;
        row = row < p.N ? row : p.N - 1;
        const u16 *src = E + (size_t)row * D + 8 * lg;
        const u16 *qsrc = qs + ln * QROW + 8 * lg;
        f32x4 dot = {0.f, 0.f, 0.f, 0.f}, gram = {0.f, 0.f, 0.f, 0.f};
#pragma unroll 4
        for (int ks = 0; ks < D / 32; ++ks) {
            const bf16x8 a = as_bf16x8(*(const v4u *)(src + ks * 32));
            const bf16x8 b = as_bf16x8(*(const v4u *)(qsrc + ks * 32));
            dot = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, dot, 0, 0, 0);
            gram = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, a, gram, 0, 0, 0);
        }
        // |e_r|^2 sits on the Gram diagonal: element (r, r) is in lane with ln == r, lg == r/4,
        // accumulator element r%4.  Lane (ln, lg) needs rows 4*lg + e.
        const float diag = (ln >> 2) == lg ? gram[ln & 3] : 0.f;
        float out[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int r = 4 * lg + e;                 // row inside the group
            const float en2 = __shfl(diag, r + 16 * (r >> 2));
            float den = sqrtf(en2) * un;
            den = den < p.eps ? p.eps : den;
            out[e] = dot[e] / den;
        }
        if (ln < p.nq_grp) {
            float *dst = p.sim + (size_t)(p.q0 + ln) * p.N + row0 + 4 * lg;
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (row0 + 4 * lg + e < p.N) dst[e] = out[e];
        }
    }
}

// One wave per context row; up to 16 queries of the group in LDS as fp32.
template <typename T>
__global__ __launch_bounds__(256) void sim_generic(GatherParams p)
{
    extern __shared__ __attribute__((aligned(16))) float qf[];   // [nq_grp][D]
    __shared__ float qnorm[16];
    const int D = p.D;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    auto ld = [](const T *ptr, size_t i) -> float {
        if constexpr (sizeof(T) == 2) return bf16_bits_to_f32(((const u16 *)ptr)[i]);
        else return ((const float *)ptr)[i];
    };
    const T *Q = (const T *)p.qry + (size_t)p.q0 * D;
    for (int idx = tid; idx < p.nq_grp * D; idx += 256) qf[idx] = ld(Q, idx);
    __syncthreads();
    for (int qi = wave; qi < p.nq_grp; qi += 4) {
        float s = 0.f;
        for (int c = lane; c < D; c += 64) s = fmaf(qf[qi * D + c], qf[qi * D + c], s);
        s = wave_sum(s);
        if (lane == 0) qnorm[qi] = sqrtf(s);
    }
    __syncthreads();
    const long stride = (long)gridDim.x * 4;
    for (long row = (long)blockIdx.x * 4 + wave; row < p.N; row += stride) {
        const T *e = (const T *)p.emb + (size_t)row * D;
        float dot[16], en2 = 0.f;
#pragma unroll
        for (int qi = 0; qi < 16; ++qi) dot[qi] = 0.f;
        for (int c = lane; c < D; c += 64) {
            const float x = ld(e, c);
            en2 = fmaf(x, x, en2);
#pragma unroll
            for (int qi = 0; qi < 16; ++qi)
                if (qi < p.nq_grp) dot[qi] = fmaf(x, qf[qi * D + c], dot[qi]);
        }
        en2 = wave_sum(en2);
#pragma unroll
        for (int qi = 0; qi < 16; ++qi) {
            if (qi < p.nq_grp) {
                const float dsum = wave_sum(dot[qi]);
                float den = sqrtf(en2) * qnorm[qi];
                den = den < p.eps ? p.eps : den;
                if (lane == 0) p.sim[(size_t)(p.q0 + qi) * p.N + row] = dsum / den;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Zero the selection histograms, the bitmap and the counters of one call.
__global__ void gather_zero(GatherParams p)
{
    const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
    const long nh = (long)p.nq * 3 * 2048;
    if (i < nh) p.hist[i] = 0;
    if (i < p.nwords) p.bitmap[i] = 0u;
}

__device__ __forceinline__ int digit_of(uint32_t u, int pass)
{
    return pass == 0 ? (int)(u >> 21) : pass == 1 ? (int)((u >> 10) & 2047u) : (int)(u & 1023u);
}
__device__ __forceinline__ bool prefix_match(uint32_t u, uint32_t prefix, int pass)
{
    return pass == 0 ? true : pass == 1 ? (u >> 21) == prefix : (u >> 10) == prefix;
}

// grid (nblk, nq): histogram of the current digit over the candidates matching the prefix.
__global__ __launch_bounds__(256) void select_hist(GatherParams p, int pass)
{
    __shared__ int h[2048];
    const int q = blockIdx.y, tid = threadIdx.x;
    for (int i = tid; i < 2048; i += 256) h[i] = 0;
    __syncthreads();
    const uint32_t prefix = pass ? p.sel_prefix[q] : 0u;
    const float *s = p.sim + (size_t)q * p.N;
    const long t0 = (long)blockIdx.x * kSelBlock;
    for (int i = tid; i < kSelBlock; i += 256) {
        const long t = t0 + i;
        if (t < p.N) {
            const uint32_t u = ordered_key(s[t]);
            if (prefix_match(u, prefix, pass)) atomicAdd(&h[digit_of(u, pass)], 1);
        }
    }
    __syncthreads();
    int *gh = p.hist + ((size_t)q * 3 + pass) * 2048;
    for (int i = tid; i < 2048; i += 256)
        if (h[i]) atomicAdd(&gh[i], h[i]);
}

// grid (nq): pick the digit holding the k-th largest, update (prefix, k remaining).
__global__ __launch_bounds__(256) void select_pick(GatherParams p, int pass)
{
    __shared__ int part[256];
    __shared__ int sel_digit, sel_krem;
    const int q = blockIdx.x, tid = threadIdx.x;
    const int *gh = p.hist + ((size_t)q * 3 + pass) * 2048;
    const int krem = pass ? p.sel_krem[q] : p.k;
    // thread t owns digits 8t..8t+7; suffix count of everything above its range
    int loc[8], sum = 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) { loc[i] = gh[8 * tid + i]; sum += loc[i]; }
    part[tid] = sum;
    __syncthreads();
    int above = 0;
    for (int t = tid + 1; t < 256; ++t) above += part[t];
    // walk own digits from the top
    int acc = above;
#pragma unroll
    for (int i = 7; i >= 0; --i) {
        const int hi = acc;           // count with digit > 8*tid+i
        acc += loc[i];
        if (hi < krem && krem <= acc) { sel_digit = 8 * tid + i; sel_krem = krem - hi; }
    }
    __syncthreads();
    if (tid == 0) {
        const uint32_t prev = pass ? p.sel_prefix[q] : 0u;
        const int bits = pass == 2 ? 10 : 11;
        p.sel_prefix[q] = (prev << bits) | (uint32_t)sel_digit;
        p.sel_krem[q] = sel_krem;
    }
}

// grid (nblk, nq): per block, how many candidates are above / equal to the threshold key.
__global__ __launch_bounds__(256) void select_count(GatherParams p)
{
    __shared__ int red[2][4];
    const int q = blockIdx.y, tid = threadIdx.x;
    const uint32_t T = p.sel_prefix[q];
    const float *s = p.sim + (size_t)q * p.N;
    const long t0 = (long)blockIdx.x * kSelBlock;
    int gt = 0, eq = 0;
    for (int i = tid; i < kSelBlock; i += 256) {
        const long t = t0 + i;
        if (t < p.N) {
            const uint32_t u = ordered_key(s[t]);
            gt += u > T;
            eq += u == T;
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

__device__ __forceinline__ int block256_excl_scan(int x, int *tmp, int &total)
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
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        const int t = tmp[w];
        if (w < wave) base += t;
        tot += t;
    }
    total = tot;
    return base + incl - x;
}

// grid (nblk, nq): ordered emission of the selected indices (ascending), lowest-index ties.
__global__ __launch_bounds__(256) void select_write(GatherParams p)
{
    __shared__ int tmp[4];
    __shared__ int sh_gt, sh_eq;
    const int q = blockIdx.y, tid = threadIdx.x, blk = blockIdx.x;
    const uint32_t T = p.sel_prefix[q];
    const int need_eq = p.sel_krem[q];
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

    const float *s = p.sim + (size_t)q * p.N;
    const long t0 = (long)blk * kSelBlock + tid * 16;
    uint32_t u[16];
    float val[16];
    int gt_c = 0, eq_c = 0;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const long t = t0 + i;
        const bool valid = t < p.N;
        val[i] = valid ? s[t] : 0.f;
        u[i] = valid ? ordered_key(val[i]) : 0u;
        gt_c += valid && u[i] > T;
        eq_c += valid && u[i] == T;
    }
    int tot;
    const int eq_before = base_eq + block256_excl_scan(eq_c, tmp, tot);
    const int eq_take = max(0, min(eq_c, need_eq - eq_before));
    const int kept_before_blk = base_gt + min(base_eq, need_eq);
    int dest = kept_before_blk + block256_excl_scan(gt_c + eq_take, tmp, tot);
    int eq_seen = eq_before;
    int32_t *oi = p.topk_idx + (size_t)q * p.k;
    float *os = p.topk_score ? p.topk_score + (size_t)q * p.k : nullptr;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
        const long t = t0 + i;
        if (t >= p.N) break;
        bool keep = u[i] > T;
        if (u[i] == T) { keep = eq_seen < need_eq; ++eq_seen; }
        if (keep && dest < p.k) {
            oi[dest] = (int32_t)t;
            if (os) os[dest] = val[i];
            ++dest;
        }
    }
}

// ------------------------------------------------------------------------------------------
// Union with dilation through a bitmap of N bits.
__device__ __forceinline__ void set_bits(uint32_t *bm, long lo, long hi)   // inclusive range
{
    for (long w = lo >> 5; w <= (hi >> 5); ++w) {
        const long b0 = w << 5;
        const int a = (int)max(lo - b0, 0L), b = (int)min(hi - b0, 31L);
        const uint32_t mask = (b - a == 31) ? 0xffffffffu : (((1u << (b - a + 1)) - 1u) << a);
        atomicOr(&bm[w], mask);
    }
}

__global__ __launch_bounds__(256) void union_mark(GatherParams p)
{
    const long i = (long)blockIdx.x * 256 + threadIdx.x;
    const long total = (long)p.nq * p.k;
    if (i < total) {
        const long t = p.topk_idx[i];
        if (t >= 0 && t < p.N)
            set_bits(p.bitmap, max(t - p.radius, 0L), min(t + (long)p.radius, p.N - 1));
    }
    // forced first / last rows: one thread per word of each range
    if (i < p.nwords) {
        const long b0 = i << 5;
        uint32_t mask = 0u;
        for (int b = 0; b < 32; ++b) {
            const long t = b0 + b;
            if (t < p.N && (t < p.n_head || t >= p.N - p.n_tail)) mask |= 1u << b;
        }
        if (mask) atomicOr(&p.bitmap[i], mask);
    }
}

__global__ __launch_bounds__(256) void union_count_words(GatherParams p)
{
    __shared__ int red[4];
    const int tid = threadIdx.x;
    int c = 0;
    for (int i = 0; i < kUnionWordsPerBlock / 256; ++i) {
        const long w = (long)blockIdx.x * kUnionWordsPerBlock + tid * (kUnionWordsPerBlock / 256) + i;
        if (w < p.nwords) c += __popc(p.bitmap[w]);
    }
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) c += __shfl_xor(c, o);
    if ((tid & 63) == 0) red[tid >> 6] = c;
    __syncthreads();
    if (tid == 0) p.word_cnt[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

__global__ __launch_bounds__(256) void union_emit(GatherParams p)
{
    __shared__ int tmp[4];
    __shared__ int sh_base;
    const int tid = threadIdx.x, blk = blockIdx.x;
    int before = 0;
    for (int b = tid; b < blk; b += 256) before += p.word_cnt[b];
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) before += __shfl_xor(before, o);
    if (tid == 0) sh_base = 0;
    __syncthreads();
    if ((tid & 63) == 0) atomicAdd(&sh_base, before);
    __syncthreads();
    constexpr int WPT = kUnionWordsPerBlock / 256;
    uint32_t w[WPT];
    int c = 0;
    const long w0 = (long)blk * kUnionWordsPerBlock + tid * WPT;
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
        w[i] = (w0 + i < p.nwords) ? p.bitmap[w0 + i] : 0u;
        c += __popc(w[i]);
    }
    int tot;
    int dest = sh_base + block256_excl_scan(c, tmp, tot);
#pragma unroll
    for (int i = 0; i < WPT; ++i) {
        uint32_t m = w[i];
        while (m) {
            const int b = __ffs(m) - 1;
            m &= m - 1;
            p.union_idx[dest++] = (int32_t)(((w0 + i) << 5) + b);
        }
    }
    if (blk == gridDim.x - 1 && tid == 255) *p.union_count = dest;
}

// ------------------------------------------------------------------------------------------
#define RF_CHECK_LAUNCH()                     \
    do {                                      \
        hipError_t e_ = hipGetLastError();    \
        if (e_ != hipSuccess) return e_;      \
    } while (0)

hipError_t gather_similarity(GatherParams p, int dtype_is_bf16, hipStream_t st)
{
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) {
        int v = 0;
        if (hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && v > 0) cus = v;
    }
    for (int q0 = 0; q0 < p.nq; q0 += 16) {
        p.q0 = q0;
        p.nq_grp = p.nq - q0 < 16 ? p.nq - q0 : 16;
        if (dtype_is_bf16 && p.D % 32 == 0 && (size_t)16 * (p.D + 8) * 2 <= 150 * 1024) {
            const size_t smem = (size_t)16 * (p.D + 8) * sizeof(u16);
            const long ngroups = (p.N + 15) / 16;
            long grid = (ngroups + 3) / 4;
            const long cap = (long)cus * 8;
            if (grid > cap) grid = cap;
            hipError_t e = hipFuncSetAttribute((const void *)sim_bf16_mfma,
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(sim_bf16_mfma, dim3((unsigned)grid), dim3(256), smem, st, p);
        } else {
            const size_t smem = (size_t)p.nq_grp * p.D * sizeof(float);
            long grid = (p.N + 3) / 4;
            const long cap = (long)cus * 16;
            if (grid > cap) grid = cap;
            if (dtype_is_bf16) {
                hipError_t e = hipFuncSetAttribute((const void *)sim_generic<u16>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL(sim_generic<u16>, dim3((unsigned)grid), dim3(256), smem, st, p);
            } else {
                hipError_t e = hipFuncSetAttribute((const void *)sim_generic<float>,
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
                if (e != hipSuccess) return e;
                hipLaunchKernelGGL(sim_generic<float>, dim3((unsigned)grid), dim3(256), smem, st, p);
            }
        }
        RF_CHECK_LAUNCH();
    }
    return hipSuccess;
}

hipError_t gather_select_union(GatherParams p, hipStream_t st)
{
    const long nzero = max((long)p.nq * 3 * 2048, (long)p.nwords);
    hipLaunchKernelGGL(gather_zero, dim3((unsigned)((nzero + 255) / 256)), dim3(256), 0, st, p);
    RF_CHECK_LAUNCH();
    const dim3 sgrid(p.nblk, p.nq);
    for (int pass = 0; pass < 3; ++pass) {
        hipLaunchKernelGGL(select_hist, sgrid, dim3(256), 0, st, p, pass);
        RF_CHECK_LAUNCH();
        hipLaunchKernelGGL(select_pick, dim3(p.nq), dim3(256), 0, st, p, pass);
        RF_CHECK_LAUNCH();
    }
    hipLaunchKernelGGL(select_count, sgrid, dim3(256), 0, st, p);
    RF_CHECK_LAUNCH();
    hipLaunchKernelGGL(select_write, sgrid, dim3(256), 0, st, p);
    RF_CHECK_LAUNCH();
    if (p.union_idx) {
        const long total = max((long)p.nq * p.k, (long)p.nwords);
        hipLaunchKernelGGL(union_mark, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, st, p);
        RF_CHECK_LAUNCH();
        const int ub = (p.nwords + kUnionWordsPerBlock - 1) / kUnionWordsPerBlock;
        hipLaunchKernelGGL(union_count_words, dim3(ub), dim3(256), 0, st, p);
        RF_CHECK_LAUNCH();
        hipLaunchKernelGGL(union_emit, dim3(ub), dim3(256), 0, st, p);
        RF_CHECK_LAUNCH();
    }
    return hipSuccess;
}

}  // namespace reform

// Gather stage (Sec. 3.3 "Identification of significant inputs" and App. C.6 "Similarity search"
// of arXiv 2506.01215): cosine similarity of query embeddings with every context embedding,
// per-query top-k with lowest-index ties, union with a +-radius neighbourhood, sorted unique.
//
//   sim_bf16_mfma   streams the [N][D] bf16 store once; 16 rows x up to 16 queries per
//                   v_mfma_f32_16x16x32_bf16; the row norms come from a second MFMA of the row
//                   tile with itself (Gram diagonal), so the VALU does no per-element work and
//                   the kernel stays HBM-bound for 16 queries.
//   sim_generic     fp32 (or odd-shaped bf16) inputs: one wave per row, fp32 FMA.
//   select_topk     (select.hip) 3-pass radix select of the k-th largest per query, then an
//                   ordered two-kernel compaction.
//   union_*         bitmap of N bits: mark dilated hits, count, emit ascending.
#include "common.h"

namespace reform {

hipError_t select_topk(const SelParams &p, hipStream_t st);



// ------------------------------------------------------------------------------------------
// 16x16x32 operand layout (wave64): A[m][k]: lane l holds m = l%16, k = 8*(l/16)..+7;
// B[k][n]: lane l holds n = l%16, same k;  C[m][n]: lane l holds n = l%16, m = 4*(l/16) + e.
//
// The kernel is a pure HBM stream (1 flop/byte for the dot products of one query, 16 for 16), so
// what matters is bytes in flight: 8 waves per workgroup share one LDS copy of the queries, and
// every wave keeps two chunks of kChunk 16-byte loads per lane outstanding (2 x 8 KB per wave,
// about 260 KB per CU) while the MFMAs of the previous chunk run.
constexpr int kSimThreads = 512;
constexpr int kChunk = 8;            // MFMA k-steps (of 32 elements) per prefetch chunk

__device__ __forceinline__ int sim_qrow(int D)   // LDS row pitch in elements: pitch % 256 B == 32 B
{
    const int rem = (2 * D) & 255;
    return D + (((32 - rem) & 255) >> 1);
}

// FULL: dim is a multiple of 32 * kChunk, so every prefetch chunk is whole and the loads and MFMAs of
// a loop trip are unconditional (the compiler can then count the loads in flight exactly).
template <bool FULL>
__global__ __launch_bounds__(kSimThreads) void sim_bf16_mfma(GatherParams p)
{
    extern __shared__ __attribute__((aligned(16))) u16 qs[];   // [16][QROW]
    __shared__ float qnorm[16];
    const int D = p.D, QROW = sim_qrow(D);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ln = lane & 15, lg = lane >> 4;
    if (p.sel.pre_zeroed && p.q0 == 0)        // the selection that follows finds its histograms cleared
        sel_clear(p.sel, (long)blockIdx.x * kSimThreads + tid, (long)gridDim.x * kSimThreads);

    // stage the (up to 16) queries of this group, zero-padded, and their norms
    const u16 *Q = (const u16 *)p.qry + (size_t)p.q0 * D;
    for (int idx = tid; idx < 16 * (D / 8); idx += kSimThreads) {
        const int r = idx / (D / 8), c8 = idx % (D / 8);
        v4u v = {0u, 0u, 0u, 0u};
        if (r < p.nq_grp) v = *(const v4u *)(Q + (size_t)r * D + c8 * 8);
        *(v4u *)(qs + r * QROW + c8 * 8) = v;
    }
    __syncthreads();
    {
        // two queries per wave, 64 lanes per query, fixed order
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const int qi = 2 * wave + h;
            float s = 0.f;
            for (int c = lane; c < D; c += 64) {
                const float x = bf16_bits_to_f32(qs[qi * QROW + c]);
                s = fmaf(x, x, s);
            }
            s = wave_sum(s);
            if (lane == 0) qnorm[qi] = sqrtf(s);
        }
    }
    __syncthreads();
    const float un = qnorm[ln];

    const long ngroups_all = (p.N + 15) / 16;
    // A workgroup streams one contiguous range of row groups (its eight waves interleaved group
    // by group): measured 1.7 % faster than handing the groups out round-robin over the grid,
    // as long as the similarity rows are not a power of two apart (the workspace pitch is skewed;
    // with a dense 2^20-float pitch the round-robin order was the faster one by 3 %).
    const long per_wg = ((ngroups_all + gridDim.x - 1) / gridDim.x + 15) / 16 * 16;
    const long ngroups = min(ngroups_all, (long)(blockIdx.x + 1) * per_wg);
    // a wave takes pairs of adjacent groups (32 rows): g, g+1, then 16 groups further on
    auto next_grp = [](long g) -> long { return (g & 1) ? g + 2 * (kSimThreads / 64) - 1 : g + 1; };
    const int nks = D / 32;                               // k-steps per row
    const int nchunks = (nks + kChunk - 1) / kChunk;
    const u16 *E = (const u16 *)p.emb;
    const u16 *qsrc = qs + ln * QROW + 8 * lg;

    long grp = (long)blockIdx.x * per_wg + 2 * wave;
    if (grp >= ngroups) return;
    auto row_ptr = [&](long g) -> const u16 * {
        long row = g * 16 + ln;
        row = row < p.N ? row : p.N - 1;
        return E + (size_t)row * D + 8 * lg;
    };
    // The wave's stream is (group, k-chunk) in row-major order over its groups grp, grp + stride,
    // ...; a load cursor runs two chunks ahead of the compute cursor, so two chunks beyond the
    // current one are always in flight.  Both cursors advance by increments only.
    v4u cur[kChunk], nx1[kChunk], nx2[kChunk];
    long l_grp = grp;                  // load cursor
    int l_ch = 0;
    const u16 *l_base = row_ptr(grp);
    auto load_next = [&](v4u (&dst)[kChunk]) {
        if (FULL) {
            // past the wave's last group the cursor stays on it: a few redundant loads instead of a branch
#pragma unroll
            for (int i = 0; i < kChunk; ++i) dst[i] = *(const v4u *)(l_base + (l_ch * kChunk + i) * 32);
            if (l_grp < ngroups && ++l_ch == nchunks) {
                const long g = next_grp(l_grp);
                l_grp = g;
                if (g < ngroups) { l_ch = 0; l_base = row_ptr(g); }
                else l_ch = nchunks - 1;
            }
            return;
        }
        if (l_grp >= ngroups) return;
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            const int ks = l_ch * kChunk + i;
            dst[i] = ks < nks ? *(const v4u *)(l_base + ks * 32) : (v4u){0u, 0u, 0u, 0u};
        }
        if (++l_ch == nchunks) {
            l_ch = 0;
            l_grp = next_grp(l_grp);
            if (l_grp < ngroups) l_base = row_ptr(l_grp);
        }
    };
    load_next(cur);
    load_next(nx1);
    f32x4 dot = {0.f, 0.f, 0.f, 0.f}, gram = {0.f, 0.f, 0.f, 0.f};
    float held[4] = {0.f, 0.f, 0.f, 0.f};
    int ch = 0;                        // compute cursor
    while (grp < ngroups) {
        load_next(nx2);
        // MFMAs of the current chunk: dot products with the queries, Gram matrix of the row tile
#pragma unroll
        for (int i = 0; i < kChunk; ++i) {
            const int ks = ch * kChunk + i;
            if (FULL || ks < nks) {
                const bf16x8 a = as_bf16x8(cur[i]);
                const bf16x8 b = as_bf16x8(*(const v4u *)(qsrc + ks * 32));
                dot = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, dot, 0, 0, 0);
                gram = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, a, gram, 0, 0, 0);
            }
        }
        if (ch + 1 == nchunks) {
            // |e_r|^2 sits on the Gram diagonal: element (r, r) is in lane with ln == r, lg == r/4,
            // accumulator element r%4.  Lane (ln, lg) needs rows 4*lg + e.
            const long row0 = grp * 16;
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
            // The results of an even group wait for its odd neighbour, so that the wave writes the
            // 128 contiguous bytes of each query row back to back (whole cache lines).
            auto store_group = [&](long r0, const float (&o)[4]) {
                float *dst = p.sim + (size_t)(p.q0 + ln) * p.sim_ld + r0 + 4 * lg;
                if (r0 + 16 <= p.N && ((p.sim_ld & 3) == 0) && ((((uintptr_t)p.sim) & 15) == 0)) {
                    // one 16-byte store per lane (r0 and 4*lg are multiples of 4); four 4-byte
                    // stores cost the kernel 15 % of its time
                    *(f32x4 *)dst = (f32x4){o[0], o[1], o[2], o[3]};
                } else {
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (r0 + 4 * lg + e < p.N) dst[e] = o[e];
                }
            };
            if (!(grp & 1) && grp + 1 < ngroups) {
#pragma unroll
                for (int e = 0; e < 4; ++e) held[e] = out[e];
            } else if (ln < p.nq_grp) {
                if (grp & 1) store_group(row0 - 16, held);
                store_group(row0, out);
            }
            dot = (f32x4){0.f, 0.f, 0.f, 0.f};
            gram = (f32x4){0.f, 0.f, 0.f, 0.f};
        }
#pragma unroll
        for (int i = 0; i < kChunk; ++i) { cur[i] = nx1[i]; nx1[i] = nx2[i]; }
        if (++ch == nchunks) { ch = 0; grp = next_grp(grp); }
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
    if (p.sel.pre_zeroed && p.q0 == 0)
        sel_clear(p.sel, (long)blockIdx.x * 256 + tid, (long)gridDim.x * 256);
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
                if (lane == 0) p.sim[(size_t)(p.q0 + qi) * p.sim_ld + row] = dsum / den;
            }
        }
    }
}

// ------------------------------------------------------------------------------------------
// Zero the bitmap of one call.
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

// One bitmap word per thread, kUnionWordsPerBlock = 256 words (8192 rows) per workgroup.
__global__ __launch_bounds__(256) void union_count_words(GatherParams p)
{
    __shared__ int red[4];
    const int tid = threadIdx.x;
    const long w = (long)blockIdx.x * kUnionWordsPerBlock + tid;
    int c = w < p.nwords ? __popc(p.bitmap[w]) : 0;
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) c += __shfl_xor(c, o);
    if ((tid & 63) == 0) red[tid >> 6] = c;
    __syncthreads();
    if (tid == 0) p.word_cnt[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

// The set bits of the workgroup's words are expanded into an LDS staging array in ascending
// order and copied out as one contiguous, coalesced block of indices.
__global__ __launch_bounds__(256) void union_emit(GatherParams p)
{
    __shared__ int32_t stage[kUnionWordsPerBlock * 32];
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
    const long w = (long)blk * kUnionWordsPerBlock + tid;
    uint32_t m = w < p.nwords ? p.bitmap[w] : 0u;
    int tot;
    int pos = block256_excl_scan(__popc(m), tmp, tot);          // synchronises: sh_base is complete after it
    const int32_t first = (int32_t)(w << 5);
    while (m) {
        stage[pos++] = first + (__ffs(m) - 1);
        m &= m - 1;
    }
    __syncthreads();
    const int base = sh_base;
    for (int i = tid; i < tot; i += 256) p.union_idx[base + i] = stage[i];
    if (blk == gridDim.x - 1 && tid == 0) *p.union_count = base + tot;
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
        if (dtype_is_bf16 && p.D % 32 == 0 && (size_t)16 * (p.D + 128) * 2 <= 150 * 1024) {
            const int rem = (2 * p.D) & 255;
            const size_t smem = (size_t)16 * (p.D + (((32 - rem) & 255) >> 1)) * sizeof(u16);
            const long ngroups = (p.N + 15) / 16;
            long grid = (ngroups + 7) / 8;
            const long cap = (long)cus * 2;
            if (grid > cap) grid = cap;
            auto kern = p.D % (32 * kChunk) == 0 ? sim_bf16_mfma<true> : sim_bf16_mfma<false>;
            hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
            if (e != hipSuccess) return e;
            hipLaunchKernelGGL(kern, dim3((unsigned)grid), dim3(kSimThreads), smem, st, p);
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
    hipError_t es = select_topk(p.sel, st);
    if (es != hipSuccess) return es;
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

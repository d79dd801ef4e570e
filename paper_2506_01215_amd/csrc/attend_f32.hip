// fp32 chunk attention + eviction score (Sec. 3.1 / Fig. 1 step 1 of arXiv 2506.01215).
//
// The fp32 configuration is the small verification workload; gfx950 has no fast fp32 matrix
// path worth tiling for it, so these kernels favour a short, exact formulation: one wave per
// attention row (two passes: row maximum, then probabilities and P.V), and one wave per key for
// the column sums.  Accurate expf/logf, fixed summation order, no atomics.
#include "common.h"

namespace reform {

constexpr int kMaxD32 = 256;

__device__ __forceinline__ float dot_row(const float *a_lds, const float *b_glb, int D)
{
    float s = 0.f;
    for (int c = 0; c < D; c += 4) {
        const float4 b = *(const float4 *)(b_glb + c);
        s = fmaf(a_lds[c + 0], b.x, s);
        s = fmaf(a_lds[c + 1], b.y, s);
        s = fmaf(a_lds[c + 2], b.z, s);
        s = fmaf(a_lds[c + 3], b.w, s);
    }
    return s;
}

// grid = Hq * Ct workgroups of one wave.
__global__ __launch_bounds__(64) void attn_fwd_f32(AttnParams p)
{
    __shared__ float qs[kMaxD32];
    __shared__ float ps[64];
    const int lane = threadIdx.x;
    const int h = blockIdx.x / p.Ct;
    const int i = blockIdx.x % p.Ct;
    const int g = h / p.G;
    const int D = p.D;
    const float *q = (const float *)p.q + (size_t)h * p.q_hs + (size_t)i * p.q_rs;
    const float *K = (const float *)p.k + (size_t)g * p.cap * D;
    const float *V = (const float *)p.v + (size_t)g * p.cap * D;
    for (int c = lane; c < D; c += 64) qs[c] = q[c];
    __syncthreads();
    const int nvis = p.M + i + 1;

    float m = -INFINITY;
    for (int j = lane; j < nvis; j += 64) m = fmaxf(m, p.scale * dot_row(qs, K + (size_t)j * D, D));
    m = wave_max(m);

    float l = 0.f;
    float o[kMaxD32 / 64] = {0.f, 0.f, 0.f, 0.f};
    for (int j0 = 0; j0 < nvis; j0 += 64) {
        const int j = j0 + lane;
        float pj = 0.f;
        if (j < nvis) pj = expf(p.scale * dot_row(qs, K + (size_t)j * D, D) - m);
        l += pj;
        __syncthreads();
        ps[lane] = pj;
        __syncthreads();
        const int cnt = min(64, nvis - j0);
        for (int jj = 0; jj < cnt; ++jj) {
            const float pw = ps[jj];
            const float *vr = V + (size_t)(j0 + jj) * D;
#pragma unroll
            for (int u = 0; u < kMaxD32 / 64; ++u) {
                const int c = lane + 64 * u;
                if (c < D) o[u] = fmaf(pw, vr[c], o[u]);
            }
        }
    }
    l = wave_sum(l);
    float *out = (float *)p.out + (size_t)h * p.o_hs + (size_t)i * p.o_rs;
#pragma unroll
    for (int u = 0; u < kMaxD32 / 64; ++u) {
        const int c = lane + 64 * u;
        if (c < D) out[c] = o[u] / l;
    }
    if (lane == 0) p.lse[(size_t)h * p.Ct + i] = m + logf(l);
}

// grid = Hkv * n workgroups of one wave: wave (g, j) sums p_ij over the observing rows of the G
// heads of the group.  Lane t takes items t, t+64, ... of the (head, row) list, so the order of
// additions depends only on (G, first row, Ct): identical keys in the cache give identical sums.
__global__ __launch_bounds__(64) void attn_score_f32(AttnParams p)
{
    __shared__ float ks[kMaxD32];
    const int lane = threadIdx.x;
    const int g = blockIdx.x / p.n;
    const int j = blockIdx.x % p.n;
    const int D = p.D;
    const float *kr = (const float *)p.k + ((size_t)g * p.cap + j) * D;
    for (int c = lane; c < D; c += 64) ks[c] = kr[c];
    __syncthreads();
    const int i_first = max(p.Ct - p.W, max(j - p.M, 0));
    const int rows = p.Ct - i_first;
    const int items = p.G * rows;
    float acc = 0.f;
    for (int it = lane; it < items; it += 64) {
        const int h = g * p.G + it / rows;
        const int i = i_first + it % rows;
        const float *q = (const float *)p.q + (size_t)h * p.q_hs + (size_t)i * p.q_rs;
        acc += expf(p.scale * dot_row(ks, q, D) - p.lse[(size_t)h * p.Ct + i]);
    }
    acc = wave_sum(acc);
    if (lane == 0) {
        float *dst = p.score + (size_t)g * p.cap + j;
        *dst = p.accumulate ? *dst + acc : acc;
    }
}

hipError_t attend_f32_forward(const AttnParams &p, hipStream_t st)
{
    hipLaunchKernelGGL(attn_fwd_f32, dim3((unsigned)p.Hq * p.Ct), dim3(64), 0, st, p);
    return hipGetLastError();
}

hipError_t attend_f32_score(const AttnParams &p, hipStream_t st)
{
    hipLaunchKernelGGL(attn_score_f32, dim3((unsigned)p.Hkv * p.n), dim3(64), 0, st, p);
    return hipGetLastError();
}

}  // namespace reform

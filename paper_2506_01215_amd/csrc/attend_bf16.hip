// bf16 chunk attention over [cache || chunk] and the eviction score, for gfx950 MFMA.
//
// Two kernels per call (Sec. 3.1 / Fig. 1 step 1 of arXiv 2506.01215 for the attention; Sec. 3.1
// and Sec. 5 for the attention-based eviction score that the method wants fused next to it):
//
//   attn_fwd_bf16    row-owned flash-style pass: out and lse.
//   attn_score_bf16  column-owned pass: score_j = sum_h sum_i exp(s_ij - lse_i).  The exact score
//                    needs the final normaliser of every row, so QK^T is formed a second time; the
//                    probabilities are never stored.
//
// Both kernels compute the TRANSPOSED logit tile  S^T = K Q^T  with v_mfma_f32_32x32x16_bf16:
// a lane then owns one query column (lane % 32) and 16 key rows, so the softmax row statistics
// are per-lane scalars (one exchange with lane ^ 32), and the probabilities are already laid out
// as the B operand of  O^T = V^T P^T  once the contraction index is permuted consistently on
// the V side (V is written into LDS transposed, with that permutation).
//
// MFMA 32x32x16 operand layout (wave64): A[m][k]: lane l holds m = l%32, k = 8*(l/32)..+7;
// B[k][n]: lane l holds n = l%32, k = 8*(l/32)..+7;  C[m][n]: lane l holds n = l%32 and, in
// accumulator element e, m = 8*(e/4) + 4*(l/32) + e%4.
#include "common.h"

namespace reform {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

__device__ __forceinline__ f32x16 mfma32(uint4 a, uint4 b, f32x16 c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_bf16x8(a), as_bf16x8(b), c, 0, 0, 0);
}

// Position of key (within a 64-key tile) inside a transposed V row in LDS.  Within each group of
// 16 keys, key 8h + 4g + r sits at 8g + 4h + r, so that lane group g = lane/32 finds the 8 keys
// whose probabilities it holds in accumulator elements 8*(t%2)..+7 as 16 contiguous bytes.
__device__ __forceinline__ int vt_pos(int key)
{
    const int k16 = key & 15;
    return (key & ~15) + ((k16 & 4) << 1) + ((k16 & 8) >> 1) + (k16 & 3);
}

// ------------------------------------------------------------------------------------------
// Forward: out, lse.  One workgroup = NW waves; a wave owns 32*QB chunk rows of one query head.
// The waves of a workgroup cover `gp` query heads of one KV group times NW/gp row slabs, so the
// K/V tiles staged in LDS serve every wave.
template <int D, int QB, int NW>
__global__ __launch_bounds__(NW * 64) void attn_fwd_bf16(AttnParams p)
{
    constexpr int NT = NW * 64;
    constexpr int KS = D / 16;           // MFMA k-steps of Q.K^T
    constexpr int DB = D / 32;           // 32-wide output blocks of P.V
    constexpr int BN = 64;               // keys per tile
    constexpr int KROW = D + 8;          // LDS row pitch (elements), 16 B pad
    constexpr int VROW = BN + 8;
    constexpr int C8 = D / 8;            // 16-byte pieces per K/V row
    constexpr int PIECES = BN * C8 / NT; // pieces of K (and keys of V) per thread per tile
    static_assert(PIECES >= 1 && PIECES <= 4, "tile/threads mismatch");
    constexpr int WROWS = 32 * QB;

    extern __shared__ __attribute__((aligned(16))) u16 smem[];
    u16 *ldsK = smem;                          // [2][BN*KROW]
    u16 *ldsV = smem + 2 * BN * KROW;          // [2][D*VROW]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int ln = lane & 31;
    const int lg = lane >> 5;

    // block -> (kv head, head subgroup, row block); heavy (late) row blocks first
    const int bid = blockIdx.x;
    const int kvh = bid % p.Hkv;
    const int rest = bid / p.Hkv;
    const int nsub = p.G / p.gp;
    const int hs = rest % nsub;
    const int rb = p.n_row_blocks - 1 - rest / nsub;
    const int slabs = NW / p.gp;
    const int head = kvh * p.G + hs * p.gp + (wave % p.gp);
    const int rwg = slabs * WROWS;
    const int w0 = rb * rwg + (wave / p.gp) * WROWS;

    const u16 *Kg = (const u16 *)p.k + (size_t)kvh * p.cap * D;
    const u16 *Vg = (const u16 *)p.v + (size_t)kvh * p.cap * D;

    // Q^T operands stay in registers for the whole pass
    uint4 qreg[QB][KS];
    {
        const u16 *Qh = (const u16 *)p.q + (size_t)head * p.q_hs;
#pragma unroll
        for (int qb = 0; qb < QB; ++qb) {
            int row = w0 + qb * 32 + ln;
            row = row < p.Ct ? row : p.Ct - 1;
            const u16 *src = Qh + (size_t)row * p.q_rs + 8 * lg;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) qreg[qb][ks] = *(const uint4 *)(src + ks * 16);
        }
    }

    const int wg_last_row = min(rb * rwg + rwg, p.Ct) - 1;
    const int ntiles = (p.M + wg_last_row) / BN + 1;
    const int wave_last_key = (w0 < p.Ct) ? p.M + min(w0 + WROWS, p.Ct) - 1 : -1;

    f32x16 o[QB][DB];
    float m_run[QB], l_run[QB];
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        m_run[qb] = -INFINITY;
        l_run[qb] = 0.f;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int e = 0; e < 16; ++e) o[qb][db][e] = 0.f;
    }

    // per-thread slice of a tile for the global -> LDS copy
    uint4 kpre[PIECES], vpre[PIECES];
    const int v_dq = tid % C8;            // which 8-wide d slice of V this thread transposes
    const int v_k0 = (tid / C8) * PIECES; // first of its PIECES consecutive keys
    auto load_tile = [&](int t) {
        const int j0 = t * BN;
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int idx = tid + NT * i;
            int row = j0 + idx / C8;
            row = row < p.n ? row : p.n - 1;
            kpre[i] = *(const uint4 *)(Kg + (size_t)row * D + (idx % C8) * 8);
            int vrow = j0 + v_k0 + i;
            vrow = vrow < p.n ? vrow : p.n - 1;
            vpre[i] = *(const uint4 *)(Vg + (size_t)vrow * D + v_dq * 8);
        }
    };
    auto store_tile = [&](int buf) {
        u16 *dk = ldsK + buf * BN * KROW;
        u16 *dv = ldsV + buf * D * VROW;
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int idx = tid + NT * i;
            *(uint4 *)(dk + (idx / C8) * KROW + (idx % C8) * 8) = kpre[i];
        }
        const int pos = vt_pos(v_k0);
#pragma unroll
        for (int dd = 0; dd < 8; ++dd) {
            // element dd of each of this thread's keys -> PIECES consecutive bf16 of row v_dq*8+dd
            u16 e[PIECES];
#pragma unroll
            for (int i = 0; i < PIECES; ++i) {
                const uint32_t w = (dd >> 1) == 0 ? vpre[i].x : (dd >> 1) == 1 ? vpre[i].y
                                   : (dd >> 1) == 2 ? vpre[i].z : vpre[i].w;
                e[i] = (dd & 1) ? (u16)(w >> 16) : (u16)(w & 0xffffu);
            }
            u16 *dst = dv + (v_dq * 8 + dd) * VROW + pos;
            if constexpr (PIECES == 4) {
                uint2 w2;
                w2.x = (uint32_t)e[0] | ((uint32_t)e[1] << 16);
                w2.y = (uint32_t)e[2] | ((uint32_t)e[3] << 16);
                *(uint2 *)dst = w2;
            } else if constexpr (PIECES == 2) {
                *(uint32_t *)dst = (uint32_t)e[0] | ((uint32_t)e[1] << 16);
            } else {
                *dst = e[0];
            }
        }
    };

    const float c = p.scale * kLog2e;

    load_tile(0);
    store_tile(0);
    if (ntiles > 1) load_tile(1);
    __syncthreads();

    for (int t = 0; t < ntiles; ++t) {
        const int buf = t & 1;
        const int j0 = t * BN;
        if (j0 <= wave_last_key) {
            const u16 *sk = ldsK + buf * BN * KROW;
            const u16 *sv = ldsV + buf * D * VROW;
            // ---- S^T = K Q^T for 64 keys x (32*QB) queries
            f32x16 s[2][QB];
#pragma unroll
            for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                for (int qb = 0; qb < QB; ++qb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) s[kb][qb][e] = 0.f;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) {
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    const uint4 a = *(const uint4 *)(sk + (kb * 32 + ln) * KROW + ks * 16 + 8 * lg);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) s[kb][qb] = mfma32(a, qreg[qb][ks], s[kb][qb]);
                }
            }
            // ---- causal mask on tiles that reach past the first row of this wave
            if (j0 + BN - 1 > p.M + w0) {
#pragma unroll
                for (int qb = 0; qb < QB; ++qb) {
                    const int lim = p.M + w0 + qb * 32 + ln - j0;   // key offset <= lim is visible
#pragma unroll
                    for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                        for (int e = 0; e < 16; ++e) {
                            const int koff = kb * 32 + 8 * (e >> 2) + 4 * lg + (e & 3);
                            if (koff > lim) s[kb][qb][e] = -INFINITY;
                        }
                }
            }
            // ---- online softmax; probabilities packed to bf16 as B operands of P.V
            uint4 pb[QB][4];
#pragma unroll
            for (int qb = 0; qb < QB; ++qb) {
                float mx = m_run[qb];
#pragma unroll
                for (int kb = 0; kb < 2; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) mx = fmaxf(mx, s[kb][qb][e]);
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float alpha = __builtin_amdgcn_exp2f((m_run[qb] - mx) * c);
                m_run[qb] = mx;
                const float mc = mx * c;
                float rs = 0.f;
#pragma unroll
                for (int kb = 0; kb < 2; ++kb) {
                    float pv[16];
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        pv[e] = __builtin_amdgcn_exp2f(fmaf(s[kb][qb][e], c, -mc));
                        rs += pv[e];
                    }
#pragma unroll
                    for (int hh = 0; hh < 2; ++hh) {
                        uint4 w;
                        w.x = pack_bf16x2(pv[8 * hh + 0], pv[8 * hh + 1]);
                        w.y = pack_bf16x2(pv[8 * hh + 2], pv[8 * hh + 3]);
                        w.z = pack_bf16x2(pv[8 * hh + 4], pv[8 * hh + 5]);
                        w.w = pack_bf16x2(pv[8 * hh + 6], pv[8 * hh + 7]);
                        pb[qb][kb * 2 + hh] = w;
                    }
                }
                l_run[qb] = l_run[qb] * alpha + rs;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int e = 0; e < 16; ++e) o[qb][db][e] *= alpha;
            }
            // ---- O^T += V^T P^T
#pragma unroll
            for (int t16 = 0; t16 < 4; ++t16) {
#pragma unroll
                for (int db = 0; db < DB; ++db) {
                    const uint4 a = *(const uint4 *)(sv + (db * 32 + ln) * VROW + t16 * 16 + 8 * lg);
#pragma unroll
                    for (int qb = 0; qb < QB; ++qb) o[qb][db] = mfma32(a, pb[qb][t16], o[qb][db]);
                }
            }
        }
        // stage tile t+1 (already in registers) into the other buffer, prefetch tile t+2
        if (t + 1 < ntiles) {
            store_tile(buf ^ 1);
            if (t + 2 < ntiles) load_tile(t + 2);
        }
        __syncthreads();
    }

    if (wave_last_key < 0) return;
    u16 *Oh = (u16 *)p.out + (size_t)head * p.o_hs;
#pragma unroll
    for (int qb = 0; qb < QB; ++qb) {
        const int row = w0 + qb * 32 + ln;
        const float l_tot = l_run[qb] + __shfl_xor(l_run[qb], 32);
        if (row >= p.Ct) continue;
        const float inv = 1.0f / l_tot;
        u16 *dst = Oh + (size_t)row * p.o_rs;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
            for (int b = 0; b < 4; ++b) {
                uint2 w;
                w.x = pack_bf16x2(o[qb][db][4 * b + 0] * inv, o[qb][db][4 * b + 1] * inv);
                w.y = pack_bf16x2(o[qb][db][4 * b + 2] * inv, o[qb][db][4 * b + 3] * inv);
                *(uint2 *)(dst + db * 32 + 8 * b + 4 * lg) = w;
            }
        if (lg == 0)
            p.lse[(size_t)head * p.Ct + row] = (m_run[qb] * c + __builtin_amdgcn_logf(l_tot)) * kLn2;
    }
}

// ------------------------------------------------------------------------------------------
// Score: a workgroup owns NW*32*KB consecutive keys of one KV head (K^T tile held in registers
// as the A operand) and streams every observing query row of the G heads of the group through
// LDS.  Per-lane partial column sums are kept for the whole pass and reduced across the 32
// query lanes once at the end, in a fixed order: no atomics, bitwise reproducible, and two cache
// rows with identical keys get identical scores.
template <int D, int KB, int NW>
__global__ __launch_bounds__(NW * 64) void attn_score_bf16(AttnParams p)
{
    constexpr int NT = NW * 64;
    constexpr int KS = D / 16;
    constexpr int QT = 64;               // query rows per LDS tile
    constexpr int QROW = D + 8;
    constexpr int C8 = D / 8;
    constexpr int PIECES = QT * C8 / NT;
    static_assert(PIECES >= 1, "tile/threads mismatch");
    constexpr int WKEYS = 32 * KB;

    __shared__ __attribute__((aligned(16))) u16 ldsQ[2][QT * QROW];
    __shared__ float ldsL[2][QT];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int ln = lane & 31;
    const int lg = lane >> 5;

    const int kvh = blockIdx.x % p.Hkv;
    const int kt = blockIdx.x / p.Hkv;
    const int j_wg = kt * (NW * WKEYS);
    const int jw = j_wg + wave * WKEYS;

    const u16 *Kg = (const u16 *)p.k + (size_t)kvh * p.cap * D;
    uint4 kreg[KB][KS];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        int key = jw + kb * 32 + ln;
        key = key < p.n ? key : p.n - 1;
        const u16 *src = Kg + (size_t)key * D + 8 * lg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kreg[kb][ks] = *(const uint4 *)(src + ks * 16);
    }

    f32x16 col[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) col[kb][e] = 0.f;

    const int i_lo = p.Ct - p.W;                         // first observing row
    const int i_first = max(i_lo, max(j_wg - p.M, 0));   // first row that both observes and sees j_wg
    const int qt0 = i_first / QT;
    const int ntq = (p.Ct + QT - 1) / QT - qt0;          // q tiles per head (>= 1 since j_wg < n)
    const int iters = p.G * ntq;
    const float c = p.scale * kLog2e;

    uint4 qpre[PIECES];
    float lpre = 0.f;
    auto load_q = [&](int it) {
        const int hh = it / ntq;
        const int i0 = (qt0 + it % ntq) * QT;
        const int head = kvh * p.G + hh;
        const u16 *Qh = (const u16 *)p.q + (size_t)head * p.q_hs;
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int idx = tid + NT * i;
            int row = i0 + idx / C8;
            row = row < p.Ct ? row : p.Ct - 1;
            qpre[i] = *(const uint4 *)(Qh + (size_t)row * p.q_rs + (idx % C8) * 8);
        }
        if (tid < QT) {
            const int row = i0 + tid;
            lpre = (row >= i_lo && row < p.Ct) ? p.lse[(size_t)head * p.Ct + row] * kLog2e : INFINITY;
        }
    };
    auto store_q = [&](int buf) {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            const int idx = tid + NT * i;
            *(uint4 *)(&ldsQ[buf][(idx / C8) * QROW + (idx % C8) * 8]) = qpre[i];
        }
        if (tid < QT) ldsL[buf][tid] = lpre;
    };

    load_q(0);
    store_q(0);
    if (iters > 1) load_q(1);
    __syncthreads();

    for (int it = 0; it < iters; ++it) {
        const int buf = it & 1;
        const int i0 = (qt0 + it % ntq) * QT;
        if (jw < p.n) {
#pragma unroll
            for (int qb = 0; qb < 2; ++qb) {
                const int r0 = i0 + qb * 32;                 // first row of this 32-row block
                if (jw > p.M + r0 + 31) continue;            // no row of the block sees any key
                f32x16 s[KB];
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) s[kb][e] = 0.f;
#pragma unroll
                for (int ks = 0; ks < KS; ++ks) {
                    const uint4 b = *(const uint4 *)(&ldsQ[buf][(qb * 32 + ln) * QROW + ks * 16 + 8 * lg]);
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb) s[kb] = mfma32(kreg[kb][ks], b, s[kb]);
                }
                const float ls = ldsL[buf][qb * 32 + ln];
                const bool need_mask = jw + WKEYS - 1 > p.M + r0;
                const int lim = p.M + r0 + ln - jw;          // key offset <= lim is visible
#pragma unroll
                for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                    for (int e = 0; e < 16; ++e) {
                        float pv = __builtin_amdgcn_exp2f(fmaf(s[kb][e], c, -ls));
                        if (need_mask) {
                            const int koff = kb * 32 + 8 * (e >> 2) + 4 * lg + (e & 3);
                            pv = koff > lim ? 0.f : pv;
                        }
                        col[kb][e] += pv;
                    }
            }
        }
        if (it + 1 < iters) {
            store_q(buf ^ 1);
            if (it + 2 < iters) load_q(it + 2);
        }
        __syncthreads();
    }

    if (jw >= p.n) return;
    float *dst = p.score + (size_t)kvh * p.cap;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int e = 0; e < 16; ++e) {
            float x = col[kb][e];
#pragma unroll
            for (int off = 16; off >= 1; off >>= 1) x += __shfl_xor(x, off);
            const int j = jw + kb * 32 + 8 * (e >> 2) + 4 * lg + (e & 3);
            if (ln == 0 && j < p.n) dst[j] = p.accumulate ? dst[j] + x : x;
        }
}

// ------------------------------------------------------------------------------------------
// Host-side launchers (called from the C-ABI file).
template <int D, int QB, int NW>
static hipError_t launch_fwd(AttnParams p, hipStream_t st)
{
    constexpr int WROWS = 32 * QB;
    int gp = 1;
    if (p.G % 4 == 0 && NW % 4 == 0) gp = 4;
    else if (p.G % 2 == 0 && NW % 2 == 0) gp = 2;
    p.gp = gp;
    const int rwg = (NW / gp) * WROWS;
    p.n_row_blocks = (p.Ct + rwg - 1) / rwg;
    const int grid = p.Hkv * (p.G / gp) * p.n_row_blocks;
    const size_t smem = sizeof(u16) * (2 * 64 * (D + 8) + 2 * D * (64 + 8));
    auto kern = attn_fwd_bf16<D, QB, NW>;
    hipError_t e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), smem, st, p);
    return hipGetLastError();
}

template <int D, int KB, int NW>
static hipError_t launch_score(AttnParams p, hipStream_t st)
{
    const int keys_wg = NW * 32 * KB;
    const int grid = p.Hkv * ((p.n + keys_wg - 1) / keys_wg);
    hipLaunchKernelGGL((attn_score_bf16<D, KB, NW>), dim3(grid), dim3(NW * 64), 0, st, p);
    return hipGetLastError();
}

hipError_t attend_bf16_forward(const AttnParams &p, hipStream_t st)
{
    if (p.D == 128) return launch_fwd<128, 1, 8>(p, st);
    return launch_fwd<64, 1, 8>(p, st);
}

hipError_t attend_bf16_score(const AttnParams &p, hipStream_t st)
{
    if (p.D == 128) return launch_score<128, 2, 4>(p, st);
    return launch_score<64, 2, 4>(p, st);
}

}  // namespace reform

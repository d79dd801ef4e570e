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
// Both kernels compute the TRANSPOSED logit tile  S^T = K Q^T: a lane then owns one query column
// and a few key rows, so the softmax row statistics are per-lane scalars (exchanged across the
// lane groups once), and the probabilities are already laid out as the B operand of
// O^T = V^T P^T  once the contraction index is permuted consistently on the V side (the V^T
// operands are fetched from a row-major V tile with gfx950's transposing LDS load, in that
// permuted key order).  Both kernels use v_mfma_f32_16x16x32_bf16 (wave64 operand layout:
// A[m][k]: lane l holds m = l%16, k = 8*(l/16)..+7;  B[k][n]: n = l%16, same k;
// C[m][n]: lane l holds n = l%16 and, in accumulator element e, m = 4*(l/16) + e).
#include "common.h"

#include <atomic>

namespace reform {

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

// ------------------------------------------------------------------------------------------
// Global -> register -> LDS staging of one 64-key K/V tile by a workgroup of NT threads: K and V
// rows are copied as they are, 16 bytes per thread and piece.  V is NOT transposed on the way in:
// the V^T operands of O^T = V^T P^T are read with ds_read_b64_tr_b16, the transposing LDS load of
// gfx950 (see lds_read_tr16 below); two plain 16-byte stores per piece replace the transposing
// 4-byte stores and their packing VALU work (about 1 % of the kernel time, and 16 VGPRs).
//
// LDS layout, measured on gfx950: a ds_read_b128 is served half a wave at a time and is free of
// bank conflicts when the 32 lanes touch 32 different 16-byte slots modulo 512 bytes.  The K
// fragment reads have 16-lane row groups (lane%16 = row, lane/16 = 16-byte piece), so a half
// wave reads 16 rows x 2 adjacent pieces: the row pitch must be an odd multiple of 32 bytes
// (288 bytes for D = 128; 272 bytes showed 3.7x the bank-conflict cycles).  The transposing V
// reads touch 16 consecutive rows x 32 bytes per instruction; the same pitch keeps them apart.
template <int D, int NT>
struct TileStage {
    static constexpr int BN = 64;
    static constexpr int KROW = D + 16;      // row pitch of both tiles, elements
    static constexpr int C8 = D / 8;
    static constexpr int PIECES = BN * C8 / NT;
    static_assert(PIECES == 1 || PIECES == 2 || PIECES == 4, "tile/threads mismatch");
    v4u kpre[PIECES], vpre[PIECES];
    uint32_t goff;                // byte offset of this thread's first piece inside a tile (global)
    uint32_t loff;                // element offset inside an LDS tile
    int row0;                     // tile-relative row of the first piece (for the clamped tail path)

    __device__ __forceinline__ void init(int tid)
    {
        row0 = tid / C8;
        goff = (uint32_t)(row0 * D + (tid % C8) * 8) * 2u;
        loff = (uint32_t)(row0 * KROW + (tid % C8) * 8);
    }
    // Kt, Vt: tile base pointers (uniform); rows_left = n - j0 (>= 1).  Piece i sits NT/C8 rows
    // further down.
    __device__ __forceinline__ void load(const u16 *Kt, const u16 *Vt, int rows_left)
    {
        const char *kb = (const char *)Kt, *vb = (const char *)Vt;
        if (rows_left >= BN) {
#pragma unroll
            for (int i = 0; i < PIECES; ++i) {
                const uint32_t off = goff + (uint32_t)(i * (NT / C8) * D * 2);
                kpre[i] = *(const v4u *)(kb + off);
                vpre[i] = *(const v4u *)(vb + off);
            }
        } else {   // ragged last tile: rows past the end repeat the last valid row
#pragma unroll
            for (int i = 0; i < PIECES; ++i) {
                const int r = row0 + i * (NT / C8);
                const int back = r < rows_left ? 0 : r - (rows_left - 1);
                const uint32_t off = goff + (uint32_t)((i * (NT / C8) - back) * D * 2);
                kpre[i] = *(const v4u *)(kb + off);
                vpre[i] = *(const v4u *)(vb + off);
            }
        }
    }
    __device__ __forceinline__ void store(u16 *dk, u16 *dv) const
    {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) {
            *(v4u *)(dk + loff + i * (NT / C8) * KROW) = kpre[i];
            *(v4u *)(dv + loff + i * (NT / C8) * KROW) = vpre[i];
        }
    }
};

// ds_read_b64_tr_b16 (gfx950).  Within each group of 16 lanes, lane r supplies the address of four
// consecutive 16-bit elements B[r][0..3]; lane i of the group receives, as element j,
// B[4*j + i/4][i%4] (established by writing element indices into LDS and reading them back).  With
// lane r = 4*j + q pointing at V[key_j][d0 + 4*q .. +3], lane i therefore receives
// V[key_0..3][d0 + i]: four keys of one d column, half of an MFMA A operand of V^T.
__device__ __forceinline__ v2u lds_read_tr16(const u16 *p)
{
    typedef short v4s __attribute__((ext_vector_type(4)));
    const v4s r = __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s *)p);
    return __builtin_bit_cast(v2u, r);
}

__device__ __forceinline__ f32x4 mfma16(v4u a, v4u b, f32x4 c)
{
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(as_bf16x8(a), as_bf16x8(b), c, 0, 0, 0);
}

// p = exp2(s*c - mc) for the 16 logits a lane holds of one query and one 64-key tile (four 16-key
// blocks x 4 keys), packed to bf16 as the two B operands of P.V (key pairs 0 and 1); returns the
// lane's partial row sum.  Plain v_add_f32 on purpose: v_dot2c_f32_bf16 was measured NOT to
// co-execute with another wave's MFMAs on gfx950, while v_fma / v_add / v_exp / v_cvt_pk do.
__device__ __forceinline__ float softmax_row(const f32x4 (&s)[4], float c, float mc, v4u (&pb)[2])
{
    float rs = 0.f;
#pragma unroll
    for (int kp = 0; kp < 2; ++kp) {
        float pv[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            pv[j] = __builtin_amdgcn_exp2f(fmaf(s[2 * kp + (j >> 2)][j & 3], c, -mc));
            rs += pv[j];
        }
        v4u w;
        w.x = pack_bf16x2(pv[0], pv[1]);
        w.y = pack_bf16x2(pv[2], pv[3]);
        w.z = pack_bf16x2(pv[4], pv[5]);
        w.w = pack_bf16x2(pv[6], pv[7]);
        pb[kp] = w;
    }
    return rs;
}

// Forward: out, lse.  One workgroup = 8 waves; a wave owns 32 chunk rows of one query head.  The
// waves of a workgroup cover `gp` query heads of one KV group times 8/gp row slabs, so the K/V
// tiles staged in LDS (two K slots, three V slots, one barrier per 64-key tile) serve every wave.
//
// MFMA shape: v_mfma_f32_16x16x32_bf16 (A[m][k]: lane l holds m = l%16, k = 8*(l/16)..+7; B[k][n]:
// n = l%16, same k; C[m][n]: n = l%16, m = 4*(l/16) + e).  Measured on gfx950 with random bf16
// operands the matrix pipe is limited by the power budget, and this shape sustains 2.03 PFLOP/s
// against 1.83 PFLOP/s for 32x32x16 (both reach 2.36-2.39 with all-zero operands): it moves half
// the accumulator data per flop.  S^T = K Q^T is formed per 16-key block and 16-query block: a lane
// owns one query column (lane % 16) of each of the wave's two query blocks and, per key block, the
// four keys 4*(lane/16)..+3; row statistics are per-lane scalars reduced over lane/16 once at
// the end, and the probabilities are already the B operand of O^T = V^T P^T: key pair kp
// contracts the 32 keys of key blocks 2*kp and 2*kp+1, lane group g = lane/16 supplying keys
// 4g..4g+3 of each, and the transposing LDS reads fetch exactly those V rows.
//
// Wall time follows the energy of the launch (the shader clock falls to about 1.95 GHz under
// this kernel with random data), so the kernel keeps the instruction count and the data
// movement per tile small:
//   - no row maximum on the fast path: probabilities are formed against the current reference
//     m_run; if a row outgrew it by more than kBigSum (or m_run is still -inf) the tile sum of
//     that row is huge / inf / NaN, and only then the whole wave recomputes with the true maximum
//     and rescales its accumulators once;
//   - scale*log2(e) folded into one v_fma per logit, v_exp_f32 directly, packed bf16 converts;
//   - tile addresses are a uniform base plus per-thread constants computed once.
constexpr float kBigSum = 65536.0f;
constexpr int kFwdWaves = 8;

template <int D>
constexpr size_t fwd_lds_bytes()
{
    return sizeof(u16) * (size_t)(5 * 64 * (D + 16));      // two K slots, three V slots
}

template <int D>
__global__ __launch_bounds__(kFwdWaves * 64, 2) void attn_fwd_bf16(AttnParams p)
{
    constexpr int NW = kFwdWaves;
    constexpr int NT = NW * 64;
    constexpr int KS = D / 32;           // MFMA k-steps of Q.K^T
    constexpr int DB = D / 16;           // 16-wide output blocks of P.V
    using Stage = TileStage<D, NT>;
    constexpr int BN = Stage::BN, KROW = Stage::KROW;
    constexpr int KTILE = BN * KROW, VTILE = BN * KROW;
    constexpr int kWin = 4;              // fragment prefetch distance (register quads)
    constexpr int NK = 4 * KS;           // K fragments per tile  (key block, k-step)
    constexpr int NV = 2 * DB;           // V^T fragments per tile (key pair, d block)

    extern __shared__ __attribute__((aligned(16))) u16 smem[];
    u16 *ldsK = smem;                          // [2][KTILE]
    u16 *ldsV = smem + 2 * KTILE;              // [3][VTILE]

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int ln = lane & 15;
    const int lg = lane >> 4;

    // block -> (kv head, head subgroup, row block); heavy (late) row blocks first
    const int bid = blockIdx.x;
    const int kvh = bid % p.Hkv;
    const int rest = bid / p.Hkv;
    const int nsub = p.G / p.gp;
    const int hs = rest % nsub;
    const int rb = p.n_row_blocks - 1 - rest / nsub;
    const int slabs = NW / p.gp;
    const int head = kvh * p.G + hs * p.gp + (wave % p.gp);
    const int rwg = slabs * 32;
    const int w0 = rb * rwg + (wave / p.gp) * 32;

    const u16 *Kg = (const u16 *)p.k + (size_t)kvh * p.cap * D;
    const u16 *Vg = (const u16 *)p.v + (size_t)kvh * p.cap * D;

    // Q^T operands of the wave's two 16-row query blocks stay in registers for the whole pass
    v4u qreg[2][KS];
    {
        const u16 *Qh = (const u16 *)p.q + (size_t)head * p.q_hs;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
            int row = w0 + 16 * nb + ln;
            row = row < p.Ct ? row : p.Ct - 1;
            const u16 *src = Qh + (size_t)row * p.q_rs + 8 * lg;
#pragma unroll
            for (int ks = 0; ks < KS; ++ks) qreg[nb][ks] = *(const v4u *)(src + ks * 32);
        }
    }

    const int wg_last_row = min(rb * rwg + rwg, p.Ct) - 1;
    const int ntiles = (p.M + wg_last_row) / BN + 1;
    const int wave_last_key = (w0 < p.Ct) ? p.M + min(w0 + 32, p.Ct) - 1 : -1;

    f32x4 o[2][DB];
    float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
#pragma unroll
    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
        for (int db = 0; db < DB; ++db) o[nb][db] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const float c = p.scale * kLog2e;
    // per-lane fragment offsets (elements) inside a K tile / V^T tile
    const int k_frag0 = ln * KROW + 8 * lg;
    const int v_frag0 = (4 * lg + (ln >> 2)) * KROW + 4 * (ln & 3);   // see lds_read_tr16

    Stage st;
    st.init(tid);
    st.load(Kg, Vg, p.n);
    st.store(ldsK, ldsV);
    if (ntiles > 1) st.load(Kg + BN * D, Vg + BN * D, p.n - BN);
    __syncthreads();

    // Two waves share a SIMD (wave w and w + NW/2), and the barrier per tile keeps them in step.
    // To make one wave's MFMAs meet the other's softmax, the waves of the upper half run their
    // O^T += V^T P^T one tile late: iteration t does P.V of tile t-1 first, then Q.K^T and the
    // softmax of tile t, keeping the probabilities in registers across the barrier.  V therefore
    // lives in three LDS slots (tile u in slot u%3), K in two.
    const bool lag = wave >= NW / 2;
    const int tl = wave_last_key >= 0 ? wave_last_key / BN : -1;      // last tile this wave needs
    v4u pb[2][2];
    int vslot = 0;                                                    // t mod 3

    auto mask_tile = [&](f32x4 (&s)[2][4], int j0) {
        if (j0 + BN - 1 > p.M + w0) {
            asm volatile("; mask path" ::: "memory");      // diagonal tiles only: keep out of line
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                const int lim = p.M + w0 + 16 * nb + ln - j0;   // key offset <= lim is visible
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (kb * 16 + 4 * lg + e > lim) s[nb][kb][e] = -INFINITY;
            }
        }
    };
    // probabilities of one tile into pb, running sums; the rare rescale is kept out of line
    auto softmax_phase = [&](f32x4 (&s)[2][4]) {
        float rs0 = softmax_row(s[0], c, m_run[0] * c, pb[0]);
        float rs1 = softmax_row(s[1], c, m_run[1] * c, pb[1]);
        if (__builtin_amdgcn_ballot_w64(!(rs0 < kBigSum) || !(rs1 < kBigSum)) != 0ull) {
            asm volatile("; rescale path" ::: "memory");
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
                float mx = s[nb][0][0];
#pragma unroll
                for (int kb = 0; kb < 4; ++kb)
#pragma unroll
                    for (int e = 0; e < 4; ++e) mx = fmaxf(mx, s[nb][kb][e]);
                mx = fmaxf(mx, __shfl_xor(mx, 16));
                mx = fmaxf(mx, __shfl_xor(mx, 32));
                const float m_new = fmaxf(mx, m_run[nb]);
                const float alpha = __builtin_amdgcn_exp2f((m_run[nb] - m_new) * c);
                m_run[nb] = m_new;
                l_run[nb] *= alpha;
#pragma unroll
                for (int db = 0; db < DB; ++db)
#pragma unroll
                    for (int e = 0; e < 4; ++e) o[nb][db][e] *= alpha;
            }
            rs0 = softmax_row(s[0], c, m_run[0] * c, pb[0]);
            rs1 = softmax_row(s[1], c, m_run[1] * c, pb[1]);
        }
        l_run[0] += rs0;
        l_run[1] += rs1;
    };

    for (int t = 0; t < ntiles; ++t) {
        const int j0 = t * BN;
        const u16 *sk = ldsK + (t & 1) * KTILE + k_frag0;
        auto kfrag = [&](int i) -> v4u {         // i = 4*ks + kb: keys 16*kb + ln, d 32*ks + 8*lg..+7
            return *(const v4u *)(sk + (i & 3) * 16 * KROW + (i >> 2) * 32);
        };
        if (!lag) {
            if (t <= tl) {
                asm volatile("; in-step wave" ::: "memory");
                const u16 *sv = ldsV + vslot * VTILE + v_frag0;
                auto vfrag = [&](int i) -> v4u { // i = DB*kp + db: d 16*db + ln, key pair kp
                    const int kp = i / DB, db = i % DB;
                    const v2u lo = lds_read_tr16(sv + (32 * kp) * KROW + 16 * db);        // keys of block 2*kp
                    const v2u hi = lds_read_tr16(sv + (32 * kp + 16) * KROW + 16 * db);   // and of block 2*kp+1
                    return (v4u){lo.x, lo.y, hi.x, hi.y};
                };
                // ---- S^T = K Q^T; fragments stream through a rolling window of kWin register
                // quads, each feeding the MFMAs of both query blocks; the window is refilled with
                // the first V^T fragments while the last MFMAs run
                v4u fw[kWin];
#pragma unroll
                for (int i = 0; i < kWin; ++i) fw[i] = kfrag(i);
                f32x4 s[2][4];
#pragma unroll
                for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                    for (int kb = 0; kb < 4; ++kb) s[nb][kb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                for (int f = 0; f < NK; ++f) {
                    s[0][f & 3] = mfma16(fw[f % kWin], qreg[0][f >> 2], s[0][f & 3]);
                    s[1][f & 3] = mfma16(fw[f % kWin], qreg[1][f >> 2], s[1][f & 3]);
                    const int g = f + kWin;
                    fw[f % kWin] = g < NK ? kfrag(g) : vfrag(g - NK);
                }
                __builtin_amdgcn_sched_group_barrier(0x100, kWin, 0);
#pragma unroll
                for (int f = 0; f < NK - kWin; ++f) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                }
#pragma unroll
                for (int f = NK - kWin; f < NK; ++f) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                    __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);   // a V^T fragment is two reads
                }
                mask_tile(s, j0);
                softmax_phase(s);
                // ---- O^T += V^T P^T, rest of the V^T fragments
#pragma unroll
                for (int f = 0; f < NV; ++f) {
                    o[0][f % DB] = mfma16(fw[f % kWin], pb[0][f / DB], o[0][f % DB]);
                    o[1][f % DB] = mfma16(fw[f % kWin], pb[1][f / DB], o[1][f % DB]);
                    if (f + kWin < NV) fw[f % kWin] = vfrag(f + kWin);
                }
#pragma unroll
                for (int f = 0; f < NV; ++f) {
                    __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                    if (f + kWin < NV) __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                }
            }
        } else {
            const bool do_pv = t >= 1 && t - 1 <= tl, do_qk = t <= tl;
            if (do_pv || do_qk) {
                asm volatile("; lagging wave" ::: "memory");
                const u16 *sv = ldsV + (vslot == 0 ? 2 : vslot - 1) * VTILE + v_frag0;   // tile t-1
                auto vfrag = [&](int i) -> v4u {
                    const int kp = i / DB, db = i % DB;
                    const v2u lo = lds_read_tr16(sv + (32 * kp) * KROW + 16 * db);
                    const v2u hi = lds_read_tr16(sv + (32 * kp + 16) * KROW + 16 * db);
                    return (v4u){lo.x, lo.y, hi.x, hi.y};
                };
                v4u fw[kWin];
                if (do_pv) {
                    // ---- O^T += V^T P^T of the previous tile; the window is refilled with the
                    // first K fragments of this tile while the last MFMAs run
#pragma unroll
                    for (int i = 0; i < kWin; ++i) fw[i] = vfrag(i);
#pragma unroll
                    for (int f = 0; f < NV; ++f) {
                        o[0][f % DB] = mfma16(fw[f % kWin], pb[0][f / DB], o[0][f % DB]);
                        o[1][f % DB] = mfma16(fw[f % kWin], pb[1][f / DB], o[1][f % DB]);
                        const int g = f + kWin;
                        fw[f % kWin] = g < NV ? vfrag(g) : kfrag(g - NV);
                    }
                    __builtin_amdgcn_sched_group_barrier(0x100, 2 * kWin, 0);
#pragma unroll
                    for (int f = 0; f < NV - kWin; ++f) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
                    }
#pragma unroll
                    for (int f = NV - kWin; f < NV; ++f) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                        __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                } else {
#pragma unroll
                    for (int i = 0; i < kWin; ++i) fw[i] = kfrag(i);
                }
                if (do_qk) {
                    f32x4 s[2][4];
#pragma unroll
                    for (int nb = 0; nb < 2; ++nb)
#pragma unroll
                        for (int kb = 0; kb < 4; ++kb) s[nb][kb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int f = 0; f < NK; ++f) {
                        s[0][f & 3] = mfma16(fw[f % kWin], qreg[0][f >> 2], s[0][f & 3]);
                        s[1][f & 3] = mfma16(fw[f % kWin], qreg[1][f >> 2], s[1][f & 3]);
                        if (f + kWin < NK) fw[f % kWin] = kfrag(f + kWin);
                    }
#pragma unroll
                    for (int f = 0; f < NK; ++f) {
                        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);
                        if (f + kWin < NK) __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
                    }
                    mask_tile(s, j0);
                    softmax_phase(s);
                }
            }
        }
        // stage tile t+1 (already in registers), prefetch tile t+2
        if (t + 1 < ntiles) {
            const int vnext = vslot == 2 ? 0 : vslot + 1;
            st.store(ldsK + ((t + 1) & 1) * KTILE, ldsV + vnext * VTILE);
            if (t + 2 < ntiles) {
                const size_t off = (size_t)(j0 + 2 * BN) * D;
                st.load(Kg + off, Vg + off, p.n - (j0 + 2 * BN));
            }
        }
        vslot = vslot == 2 ? 0 : vslot + 1;
        __syncthreads();
    }
    if (lag && tl == ntiles - 1) {
        // the lagging waves still owe the P.V of their last tile (slot (ntiles-1) % 3)
        const u16 *sv = ldsV + (vslot == 0 ? 2 : vslot - 1) * VTILE + v_frag0;
#pragma unroll
        for (int f = 0; f < NV; ++f) {
            const int kp = f / DB, db = f % DB;
            const v2u lo = lds_read_tr16(sv + (32 * kp) * KROW + 16 * db);
            const v2u hi = lds_read_tr16(sv + (32 * kp + 16) * KROW + 16 * db);
            const v4u a = {lo.x, lo.y, hi.x, hi.y};
            o[0][db] = mfma16(a, pb[0][kp], o[0][db]);
            o[1][db] = mfma16(a, pb[1][kp], o[1][db]);
        }
    }

    if (wave_last_key < 0) return;
    u16 *Oh = (u16 *)p.out + (size_t)head * p.o_hs;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
        const int row = w0 + 16 * nb + ln;
        float l_tot = l_run[nb] + __shfl_xor(l_run[nb], 16);
        l_tot += __shfl_xor(l_tot, 32);
        if (row >= p.Ct) continue;
        const float inv = 1.0f / l_tot;
        u16 *dst = Oh + (size_t)row * p.o_rs;
#pragma unroll
        for (int db = 0; db < DB; ++db) {
            v2u w;
            w.x = pack_bf16x2(o[nb][db][0] * inv, o[nb][db][1] * inv);
            w.y = pack_bf16x2(o[nb][db][2] * inv, o[nb][db][3] * inv);
            *(v2u *)(dst + db * 16 + 4 * lg) = w;
        }
        if (lg == 0) p.lse[(size_t)head * p.Ct + row] = (m_run[nb] * c + __builtin_amdgcn_logf(l_tot)) * kLn2;
    }
}

// ------------------------------------------------------------------------------------------
// Score: a workgroup owns NW*16*KB consecutive keys of one KV head (K^T tile held in registers
// as the A operand) and streams every observing query row of the G heads of the group through
// LDS.  Per-lane partial column sums are kept for the whole pass and reduced across the 16
// query lanes once at the end, in a fixed order: no atomics, bitwise reproducible, and two cache
// rows with identical keys get identical scores.
//
// Per logit the VALU does one v_fma (scale and -lse folded), one v_exp and one v_add; the mask is
// applied only on the tiles that straddle the causal diagonal (separate, rarely taken path), and
// rows outside the observation window or past the chunk end are switched off through lse = +inf.
template <int D, int NT>
struct QStage {
    static constexpr int QT = 64;
    static constexpr int QROW = D + 16;
    static constexpr int C8 = D / 8;
    static constexpr int PIECES = QT * C8 / NT;
    static_assert(PIECES >= 1, "tile/threads mismatch");
    v4u qpre[PIECES];
    float lpre;
    bool lvalid;
    uint32_t goff, gstep;     // byte offset of this thread's first piece inside a tile, step per piece
    uint32_t loff;            // element offset inside the LDS tile
    int row0;

    __device__ __forceinline__ void init(int tid, long q_rs)
    {
        row0 = tid / C8;
        goff = (uint32_t)((long)row0 * q_rs * 2 + (tid % C8) * 16);
        gstep = (uint32_t)((long)(NT / C8) * q_rs * 2);
        loff = (uint32_t)(row0 * QROW + (tid % C8) * 8);
        lpre = 0.f;
        lvalid = false;
    }
    // Qt: first row of the tile (uniform); lse_t: lse of that row; rows_left = Ct - i0 (>= 1);
    // first_obs = first observing row relative to the tile (<= 0 when the whole tile observes)
    __device__ __forceinline__ void load(const u16 *Qt, const float *lse_t, int rows_left, int first_obs,
                                         long q_rs, int tid)
    {
        const char *qb = (const char *)Qt;
        if (rows_left >= QT) {
#pragma unroll
            for (int i = 0; i < PIECES; ++i) qpre[i] = *(const v4u *)(qb + (goff + gstep * (uint32_t)i));
        } else {
#pragma unroll
            for (int i = 0; i < PIECES; ++i) {
                int r = row0 + i * (NT / C8);
                r = r < rows_left ? r : rows_left - 1;
                qpre[i] = *(const v4u *)(qb + ((size_t)r * q_rs * 2 + (tid % C8) * 16));
            }
        }
        // raw value only: multiplying here would wait for the load right after issuing it
        if (tid < QT) {
            lvalid = tid >= first_obs && tid < rows_left;
            lpre = lvalid ? lse_t[tid] : 0.f;
        }
    }
    __device__ __forceinline__ void store(u16 *dq, float *dl, int tid) const
    {
#pragma unroll
        for (int i = 0; i < PIECES; ++i) *(v4u *)(dq + loff + i * (NT / C8) * QROW) = qpre[i];
        if (tid < QT) dl[tid] = lvalid ? lpre * kLog2e : INFINITY;
    }
};

// A wave holds 64 keys (four 16-key blocks) as A operands for the whole pass; query rows stream
// through LDS as B operands, two 16-row blocks at a time; a lane owns one query column of each
// block and 4 keys per key block.  The MFMA shape and the operand order were chosen by
// measurement under the power cap (random bf16 operands): 16x16x32 sustains 2.03 PFLOP/s in a
// pure MFMA loop against 1.83 for 32x32x16, and an A operand that is held for two MFMAs while B
// alternates between two registers costs 4 % less than a new A operand on every MFMA.  The
// 32x32x16 form of this kernel (32 keys x 32 rows per MFMA, new key fragment every MFMA) was
// 1.2 % slower.
template <int D, int KB, int NW>
__global__ __launch_bounds__(NW * 64, 2) void attn_score_bf16(AttnParams p)
{
    constexpr int NT = NW * 64;
    constexpr int KS = D / 32;                           // MFMA k-steps
    using Stage = QStage<D, NT>;
    constexpr int QT = Stage::QT, QROW = Stage::QROW;
    constexpr int WKEYS = 16 * KB;
    constexpr int NQB = QT / 16;                         // 16-row query blocks per tile
    static_assert(NQB % 4 == 0, "the rotation below alternates two units of two query blocks");

    __shared__ __attribute__((aligned(16))) u16 ldsQ[2][QT * QROW];
    __shared__ float ldsL[2][QT];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int ln = lane & 15;
    const int lg = lane >> 4;

    const int kvh = blockIdx.x % p.Hkv;
    const int kt = blockIdx.x / p.Hkv;
    const int j_wg = kt * (NW * WKEYS);
    const int jw = j_wg + wave * WKEYS;

    const u16 *Kg = (const u16 *)p.k + (size_t)kvh * p.cap * D;
    v4u kreg[KB][KS];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) {
        int key = jw + kb * 16 + ln;
        key = key < p.n ? key : p.n - 1;
        const u16 *src = Kg + (size_t)key * D + 8 * lg;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) kreg[kb][ks] = *(const v4u *)(src + ks * 32);
    }

    f32x4 col[KB];
#pragma unroll
    for (int kb = 0; kb < KB; ++kb) col[kb] = (f32x4){0.f, 0.f, 0.f, 0.f};

    const int i_lo = p.Ct - p.W;                         // first observing row
    const int i_first = max(i_lo, max(j_wg - p.M, 0));   // first row that both observes and sees j_wg
    const int qt0 = i_first / QT;
    const int ntq = (p.Ct + QT - 1) / QT - qt0;          // q tiles per head (>= 1 since j_wg < n)
    const int iters = p.G * ntq;
    const float c = p.scale * kLog2e;
    const int q_frag0 = ln * QROW + 8 * lg;

    Stage st;
    st.init(tid, p.q_rs);
    auto load_q = [&](int it) {
        const int head = kvh * p.G + it / ntq;
        const int i0 = (qt0 + it % ntq) * QT;
        st.load((const u16 *)p.q + (size_t)head * p.q_hs + (size_t)i0 * p.q_rs,
                p.lse + (size_t)head * p.Ct + i0, p.Ct - i0, i_lo - i0, p.q_rs, tid);
    };
    load_q(0);
    st.store(ldsQ[0], ldsL[0], tid);
    if (iters > 1) load_q(1);
    __syncthreads();

    // Rotation inside a wave, in units of two adjacent 16-row query blocks: the 32 MFMAs of a unit
    // are interleaved, one MFMA to three VALU instructions, with the v_fma / v_exp / v_add work of
    // the PREVIOUS unit, which never waits for the MFMAs in flight.  Every key fragment (A
    // operand) is used for two MFMAs in a row, the B operand alternating between the unit's two
    // query blocks.  `sB` / `lsB0`, `lsB1` carry the unit whose VALU work is pending; lse = +inf
    // makes a block contribute exactly 0 (the empty state).
    f32x4 sA[2][KB], sB[2][KB];
#pragma unroll
    for (int h = 0; h < 2; ++h)
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) sB[h][kb] = (f32x4){0.f, 0.f, 0.f, 0.f};
    float lsB0 = INFINITY, lsB1 = INFINITY;
    auto issue_mfma2 = [&](f32x4 (&dst)[2][KB], const u16 *src) {
        v4u bq0[KS], bq1[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            bq0[ks] = *(const v4u *)(src + ks * 32);
            bq1[ks] = *(const v4u *)(src + 16 * QROW + ks * 32);
        }
#pragma unroll
        for (int h = 0; h < 2; ++h)
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) dst[h][kb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) {
                dst[0][kb] = mfma16(kreg[kb][ks], bq0[ks], dst[0][kb]);
                dst[1][kb] = mfma16(kreg[kb][ks], bq1[ks], dst[1][kb]);
            }
    };
    auto accumulate2 = [&](const f32x4 (&src)[2][KB], float ls0, float ls1) {
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                col[kb][e] += __builtin_amdgcn_exp2f(fmaf(src[0][kb][e], c, -ls0));
                col[kb][e] += __builtin_amdgcn_exp2f(fmaf(src[1][kb][e], c, -ls1));
            }
    };
    f32x4 sD[KB];                          // diagonal path: one 16-row block at a time
    auto issue_mfma = [&](f32x4 (&dst)[KB], const u16 *src) {
        v4u bq[KS];
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) bq[ks] = *(const v4u *)(src + ks * 32);
#pragma unroll
        for (int kb = 0; kb < KB; ++kb) dst[kb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
#pragma unroll
            for (int kb = 0; kb < KB; ++kb) dst[kb] = mfma16(kreg[kb][ks], bq[ks], dst[kb]);
    };
    auto interleave_pattern = [&]() {
        __builtin_amdgcn_sched_group_barrier(0x100, 2 * KS, 0);
#pragma unroll
        for (int u = 0; u < 2 * KS * KB; ++u) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);     // one MFMA ...
            __builtin_amdgcn_sched_group_barrier(0x402, 3, 0);     // ... then three VALU/transcendental ops
        }
    };
    for (int it = 0; it < iters; ++it) {
        const int buf = it & 1;
        const int i0 = (qt0 + it % ntq) * QT;
        if (jw < p.n) {
            const u16 *sq = ldsQ[buf] + q_frag0;
            if (jw + WKEYS - 1 <= p.M + i0) {
                // ---- every row of the tile sees every key of this wave
#pragma unroll
                for (int qb = 0; qb < NQB; qb += 4) {
                    const float l0 = ldsL[buf][16 * qb + ln], l1 = ldsL[buf][16 * qb + 16 + ln];
                    const float l2 = ldsL[buf][16 * qb + 32 + ln], l3 = ldsL[buf][16 * qb + 48 + ln];
                    issue_mfma2(sA, sq + 16 * qb * QROW);
                    accumulate2(sB, lsB0, lsB1);
                    interleave_pattern();
                    __builtin_amdgcn_sched_barrier(0);
                    issue_mfma2(sB, sq + (16 * qb + 32) * QROW);
                    accumulate2(sA, l0, l1);
                    interleave_pattern();
                    __builtin_amdgcn_sched_barrier(0);
                    lsB0 = l2;
                    lsB1 = l3;
                }
            } else {
                asm volatile("; diagonal path" ::: "memory");
                accumulate2(sB, lsB0, lsB1);          // flush the pending unit first
                lsB0 = INFINITY;
                lsB1 = INFINITY;
#pragma unroll 1
                for (int qb = 0; qb < NQB; ++qb) {
                    const int r0 = i0 + qb * 16;                 // first row of this 16-row block
                    if (jw > p.M + r0 + 15) continue;            // no row of the block sees any key
                    issue_mfma(sD, sq + qb * 16 * QROW);
                    const float ls = ldsL[buf][qb * 16 + ln];
                    const int lim = p.M + r0 + ln - jw;          // key offset <= lim is visible
#pragma unroll
                    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
                        for (int e = 0; e < 4; ++e) {
                            const int koff = kb * 16 + 4 * lg + e;
                            const float pv = __builtin_amdgcn_exp2f(fmaf(sD[kb][e], c, -ls));
                            col[kb][e] += koff > lim ? 0.f : pv;
                        }
                }
            }
        }
        if (it + 1 < iters) {
            st.store(ldsQ[buf ^ 1], ldsL[buf ^ 1], tid);
            if (it + 2 < iters) load_q(it + 2);
        }
        __syncthreads();
    }
    accumulate2(sB, lsB0, lsB1);               // flush the last pending unit

    if (jw >= p.n) return;
    float *dst = p.score + (size_t)kvh * p.cap;
#pragma unroll
    for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            float x = col[kb][e];
#pragma unroll
            for (int off = 8; off >= 1; off >>= 1) x += __shfl_xor(x, off);    // over the 16 query lanes
            const int j = jw + kb * 16 + 4 * lg + e;
            if (ln == 0 && j < p.n) dst[j] = p.accumulate ? dst[j] + x : x;
        }
}

// ------------------------------------------------------------------------------------------
// Host-side launchers (called from the C-ABI file).
template <int D>
static hipError_t launch_fwd(AttnParams p, hipStream_t st)
{
    constexpr int NW = kFwdWaves;
    int gp = 1;
    if (p.G % 4 == 0) gp = 4;
    else if (p.G % 2 == 0) gp = 2;
    p.gp = gp;
    const int rwg = (NW / gp) * 32;
    p.n_row_blocks = (p.Ct + rwg - 1) / rwg;
    const int grid = p.Hkv * (p.G / gp) * p.n_row_blocks;
    const size_t smem = fwd_lds_bytes<D>();
    auto kern = attn_fwd_bf16<D>;
    // the kernel needs more than the default 64 KB of LDS: raised once per device, not per launch
    static std::atomic<bool> lds_raised[64];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 64 || !lds_raised[dev].load(std::memory_order_acquire)) {
        e = hipFuncSetAttribute((const void *)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        if (dev >= 0 && dev < 64) lds_raised[dev].store(true, std::memory_order_release);
    }
    hipLaunchKernelGGL(kern, dim3(grid), dim3(NW * 64), smem, st, p);
    return hipGetLastError();
}

template <int D, int KB, int NW>
static hipError_t launch_score(AttnParams p, hipStream_t st)
{
    const int keys_wg = NW * 16 * KB;
    const int grid = p.Hkv * ((p.n + keys_wg - 1) / keys_wg);
    hipLaunchKernelGGL((attn_score_bf16<D, KB, NW>), dim3(grid), dim3(NW * 64), 0, st, p);
    return hipGetLastError();
}

hipError_t attend_bf16_forward(const AttnParams &p, hipStream_t st)
{
    if (p.D == 128) return launch_fwd<128>(p, st);
    return launch_fwd<64>(p, st);
}

hipError_t attend_bf16_score(const AttnParams &p, hipStream_t st)
{
    if (p.D == 128) return launch_score<128, 4, 8>(p, st);
    return launch_score<64, 4, 4>(p, st);
}

}  // namespace reform

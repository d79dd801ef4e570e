// Shared device helpers and launch-parameter structs of the gfx950 kernels.
// Nothing here is shared with the CPU oracle.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace reform {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef unsigned short u16;
// 16-byte register quad as a native vector (HIP's uint4 is a struct whose copies lower to
// memcpy and can strand small arrays in scratch memory).
typedef unsigned int v4u __attribute__((ext_vector_type(4)));
typedef unsigned int v2u __attribute__((ext_vector_type(2)));

constexpr int kWave = 64;

struct AttnParams {
    const void *q, *k, *v;
    void *out;
    float *lse;      // never null inside the kernels (caller's buffer or workspace)
    float *score;    // may be null for the forward kernel
    int Hq, Hkv, G, D;
    int M, Ct, cap, n;
    long q_hs, q_rs, o_hs, o_rs;
    float scale;
    int W;           // resolved observation window, 1..Ct
    int accumulate;
    int gp;          // query heads of one group that share a workgroup (1, 2 or 4)
    int n_row_blocks;
};

#ifndef RF_MOVE_TILE
#define RF_MOVE_TILE 16384
#endif
constexpr int kMoveTileBytes = RF_MOVE_TILE;   // bytes of destination rows per workgroup of the in-place move
constexpr int kUnionWordsPerBlock = 256;   // bitmap words per workgroup of the union kernels

// Top-k selection problem: nq rows of N candidates (row stride ld), k winners per row.
struct SelParams {
    const float *vals;
    long ld, N;
    int nq, k;
    int n_sink, n_recent;    // first / last slots that are always selected (count inside k)
    int *hist;               // [nq][3][2048]
    uint32_t *sel_prefix;    // [3][nq]  selection state after each radix pass
    int *sel_krem;           // [3][nq]
    int *blk_cnt;            // [nq][nblk][2]   (above, equal) per workgroup
    int nblk;                // ceil(N / 4096)
    int32_t *out_idx;        // [nq][out_ld], ascending
    float *out_val;          // nullable, values of the selected candidates
    long out_ld;
    int32_t *out_rank;       // nullable [nq][ld]: rank[t] = number of selected candidates below t
    const int32_t *side_src; // nullable [nq][ld]: a 4-byte companion of every candidate ...
    int32_t *side_dst;       // ... copied to [nq][out_ld] for the selected ones (same order as out_idx)
    int *zero_extra;         // nullable: zero_extra_n more ints cleared by the histogram-clearing launch
    int zero_extra_n;
    int pre_zeroed;          // hist and zero_extra were cleared by an earlier kernel of the same call
    int multi_ok;            // rows too long for one workgroup may be selected in one launch by several
                             // workgroups that wait for each other (needs hist, blk_cnt and err to be usable
                             // for that: the eviction sets it)
    int *err;                // nullable: set to 1 if a bounded wait between workgroups expired
    int spin_limit;          // polls of such a wait
};

struct EvictParams {
    void *k, *v;
    float *score;
    int32_t *pos;
    int32_t *kept;      // [Hkv][B]
    void *stage_k, *stage_v;   // [Hkv][B][row_bytes]
    float *stage_score;        // [Hkv][B]
    int32_t *stage_pos;        // [Hkv][B]
    SelParams sel;             // top-B over score
    int *sync;                 // in-place move: error word, per-stream tickets, per-tile flags; null = staged move
    int ntile;                 // tiles per stream of the in-place move
    int spin_limit;            // polls a tile spends on another tile's flag before giving up (0: see the kernel)
    int Hkv, n, B, cap, n_sink, n_recent;
    int row_bytes;      // head_dim * sizeof(element), multiple of 16
};

struct RowsParams {
    const void *table;       // [n_table][row_bytes]
    void *out;               // [n_idx][row_bytes]
    const int32_t *idx;      // [n_idx]
    const int32_t *count;    // nullable device scalar: only the first min(*count, n_idx) indices are used
    int *err;                // nullable device word, bit 0 set if an index was outside the table
    long n_table, n_idx, row_bytes, pieces;
};

struct RopeParams {
    void *k;                 // [Hkv][cap][d], rows [0, n_rows) already compacted
    const int32_t *kept;     // [Hkv][kept_ld]: slot each row came from
    long n_rows, cap, kept_ld;
    int Hkv, rot;            // rot: rotated leading elements of a row (even)
    int row_bytes;
    double neg2_log2_theta_over_rot;   // -2 log2(theta) / rot
};

struct EmbedParams {
    const void *src;     // first token's head vector
    void *emb;           // embedding row of the first token
    long n_rows;
    long src_stride_bytes, emb_stride_bytes, col_bytes;
    long src_head_bytes, head_bytes;   // per head (blockIdx.y): source offset, column offset
    int n_heads;
    int pieces, group;   // 16-byte pieces per head vector; lanes per row (power of two >= pieces, <= 64)
    float eps;
};

struct PoolParams {
    const float *sim;    // [nq][ld]
    float *pooled;       // [N]
    SelParams sel;       // budget selection over pooled (one row)
    long N, ld;
    int nq, window;      // window odd, <= the kernel's maximum
};

struct GatherParams {
    const void *emb, *qry;
    float *sim;          // [nq][sim_ld]
    long sim_ld;         // row pitch of sim in floats (>= N)
    int32_t *topk_idx;   // [nq][k]
    float *topk_score;   // nullable
    int32_t *union_idx;  // nullable
    int32_t *union_count;
    SelParams sel;       // per-query top-k over sim
    uint32_t *bitmap;    // [nwords]
    int *word_cnt;       // [n_union_blocks]
    long N;
    int D, nq, k, radius, n_head, n_tail;
    int nwords;          // bitmap words
    float eps;
    int q0, nq_grp;      // query group handled by this similarity launch
};

__device__ __forceinline__ float bf16_bits_to_f32(u16 b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16 bits, round to nearest even (finite inputs; NaN stays NaN).
__device__ __forceinline__ u16 f32_to_bf16_bits(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (u16)((u >> 16) | 0x40);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (u16)(u >> 16);
}

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
    typedef float f32x2 __attribute__((ext_vector_type(2)));
    f32x2 v = {lo, hi};
    bf16x2 r = __builtin_convertvector(v, bf16x2);   // v_cvt_pk_bf16_f32 on gfx950 (RNE)
    return __builtin_bit_cast(uint32_t, r);
}

__device__ __forceinline__ bf16x8 as_bf16x8(v4u v) { return __builtin_bit_cast(bf16x8, v); }

__device__ __forceinline__ float wave_sum(float x)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x += __shfl_xor(x, o);
    return x;
}
__device__ __forceinline__ float wave_max(float x)
{
#pragma unroll
    for (int o = 32; o >= 1; o >>= 1) x = fmaxf(x, __shfl_xor(x, o));
    return x;
}

// Monotone map float -> uint32: a > b  <=>  key(a) > key(b) (finite values; -0 and +0 map alike).
__device__ __forceinline__ uint32_t ordered_key(float f)
{
    uint32_t u = __float_as_uint(f);
    if (u == 0x80000000u) u = 0u;
    return (u & 0x80000000u) ? ~u : (u | 0x80000000u);
}

// Clears the selection's histograms and extra ints; thread i0 of `stride` threads.  Called at the
// start of a kernel that runs before the selection in the same library call, which saves the
// selection its own clearing launch.
__device__ __forceinline__ void sel_clear(const SelParams &p, long i0, long stride)
{
    const long nh = (long)p.nq * 3 * 2048;
    for (long i = i0; i < nh; i += stride) p.hist[i] = 0;
    for (long i = i0; i < p.zero_extra_n; i += stride) p.zero_extra[i] = 0;
    if (p.multi_ok)
        for (long i = i0; i < (long)p.nq * p.nblk * 2; i += stride) p.blk_cnt[i] = 0;
    if (p.err && i0 == 0) *p.err = 0;
}

// Exclusive scan of one int per thread over a 256-thread workgroup (tmp: 4 ints of LDS);
// returns the exclusive prefix, `total` receives the workgroup sum.
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

}  // namespace reform

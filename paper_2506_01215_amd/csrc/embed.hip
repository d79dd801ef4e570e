// Cross-layer context embedding construction (arXiv 2506.01215, Sec. 3.2 "Combining multiple
// heads": e_comb = concat{ e_i / ||e_i|| : i in selected heads }; Alg. 1 `emb.SaveSelected(qkv)`).
// One call writes the segments of the selected heads of one tensor (grid.y = head): a head's
// Q, K or V state of every token of a chunk, L2-normalised (norm clamped from below by eps, so a
// zero vector stays zero), into columns [col + h*d, col + (h+1)*d) of the tokens' rows of the
// [N][D] embedding store.
//
// Pure streaming: a group of d/(16 bytes) lanes owns a row (16 lanes for a 128-wide bf16 head, so
// a wave normalises four rows at once), one 16-byte load and one 16-byte store per lane, the
// sum of squares reduced inside the group with shuffles.  Sums are fp32.
#include "common.h"

namespace reform {

template <bool BF16>
__global__ __launch_bounds__(256) void embed_normalise_rows(EmbedParams p)
{
    // p.group = lanes per row (power of two, >= pieces per row); p.pieces = 16-byte pieces per row
    const int lane_in_grp = threadIdx.x & (p.group - 1);
    const long row = ((long)blockIdx.x * 256 + threadIdx.x) / p.group;
    const bool active = row < p.n_rows && lane_in_grp < p.pieces;
    v4u raw = {0u, 0u, 0u, 0u};
    const size_t hsrc = (size_t)blockIdx.y * p.src_head_bytes, hcol = (size_t)blockIdx.y * p.head_bytes;
    if (active)
        raw = *(const v4u *)((const char *)p.src + hsrc + (size_t)row * p.src_stride_bytes + lane_in_grp * 16);
    float x[8];
    if (BF16) {
        const uint32_t w[4] = {raw.x, raw.y, raw.z, raw.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x[2 * i] = __uint_as_float(w[i] << 16);
            x[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
        }
    } else {
        x[0] = __uint_as_float(raw.x); x[1] = __uint_as_float(raw.y);
        x[2] = __uint_as_float(raw.z); x[3] = __uint_as_float(raw.w);
        x[4] = x[5] = x[6] = x[7] = 0.f;
    }
    float ss = 0.f;
#pragma unroll
    for (int i = 0; i < 8; ++i) ss = fmaf(x[i], x[i], ss);
    for (int off = p.group >> 1; off >= 1; off >>= 1) ss += __shfl_xor(ss, off);
    const float inv = 1.0f / fmaxf(sqrtf(ss), p.eps);
    if (!active) return;
    v4u o;
    if (BF16) {
        o.x = pack_bf16x2(x[0] * inv, x[1] * inv);
        o.y = pack_bf16x2(x[2] * inv, x[3] * inv);
        o.z = pack_bf16x2(x[4] * inv, x[5] * inv);
        o.w = pack_bf16x2(x[6] * inv, x[7] * inv);
    } else {
        o.x = __float_as_uint(x[0] * inv); o.y = __float_as_uint(x[1] * inv);
        o.z = __float_as_uint(x[2] * inv); o.w = __float_as_uint(x[3] * inv);
    }
    *(v4u *)((char *)p.emb + (size_t)row * p.emb_stride_bytes + p.col_bytes + hcol + lane_in_grp * 16) = o;
}

hipError_t embed_save(const EmbedParams &p, bool bf16, hipStream_t st)
{
    if (p.n_rows == 0) return hipSuccess;
    const long threads = p.n_rows * p.group;
    const unsigned grid = (unsigned)((threads + 255) / 256);
    if (bf16) hipLaunchKernelGGL(embed_normalise_rows<true>, dim3(grid, p.n_heads), dim3(256), 0, st, p);
    else hipLaunchKernelGGL(embed_normalise_rows<false>, dim3(grid, p.n_heads), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace reform

// Position reassignment after compression (arXiv 2506.01215, Sec. 3.1: after compression the
// tokens of the compressed cache get consecutive position ids).  The cache stores rotary-embedded
// keys; the key now at slot r came from slot kept[r] and is rotated by delta = r - kept[r]
// positions (half-split pairing: element c with element c + rot/2, frequency theta^(-2c/rot);
// elements beyond `rot` are left alone).  Rows that did not move (a prefix) are skipped.
//
// A thread owns one 16-byte piece of the low half of a row and the matching piece of the high
// half.  The angle delta * theta^(-2c/rot) reaches tens of thousands of radians, so it is formed
// and reduced to a fraction of a turn in fp64; sine and cosine of the reduced angle are fp32.
#include "common.h"

namespace reform {

template <bool BF16>
__global__ __launch_bounds__(256) void rope_rerotate(RopeParams p)
{
    constexpr int E = BF16 ? 8 : 4;                      // elements per 16-byte piece
    const int tpr = p.rot / (2 * E);                     // threads per row
    const long gid = (long)blockIdx.x * 256 + threadIdx.x;
    const long row = gid / tpr;
    const int piece = (int)(gid % tpr);
    const int g = blockIdx.y;
    if (row >= p.n_rows) return;
    const int delta = (int)row - p.kept[(size_t)g * p.kept_ld + row];
    if (delta == 0) return;
    char *base = (char *)p.k + ((size_t)g * p.cap + row) * p.row_bytes;
    v4u *plo = (v4u *)(base + piece * 16);
    v4u *phi = (v4u *)(base + (p.rot / 2) * (BF16 ? 2 : 4) + piece * 16);
    const v4u lo = *plo, hi = *phi;
    float x0[E], x1[E];
    if (BF16) {
        const uint32_t a[4] = {lo.x, lo.y, lo.z, lo.w}, b[4] = {hi.x, hi.y, hi.z, hi.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            x0[2 * i] = __uint_as_float(a[i] << 16);
            x0[2 * i + 1] = __uint_as_float(a[i] & 0xffff0000u);
            x1[2 * i] = __uint_as_float(b[i] << 16);
            x1[2 * i + 1] = __uint_as_float(b[i] & 0xffff0000u);
        }
    } else {
        x0[0] = __uint_as_float(lo.x); x0[1] = __uint_as_float(lo.y);
        x0[2] = __uint_as_float(lo.z); x0[3] = __uint_as_float(lo.w);
        x1[0] = __uint_as_float(hi.x); x1[1] = __uint_as_float(hi.y);
        x1[2] = __uint_as_float(hi.z); x1[3] = __uint_as_float(hi.w);
    }
    float y0[E], y1[E];
#pragma unroll
    for (int i = 0; i < E; ++i) {
        const int c = piece * E + i;
        const double turns = (double)delta * exp2(p.neg2_log2_theta_over_rot * (double)c) * 0.15915494309189535;
        const float frac = (float)(turns - rint(turns));           // in [-0.5, 0.5]
        float sn, cs;
        sincosf(frac * 6.2831853071795865f, &sn, &cs);
        y0[i] = x0[i] * cs - x1[i] * sn;
        y1[i] = x1[i] * cs + x0[i] * sn;
    }
    v4u olo, ohi;
    if (BF16) {
        olo.x = pack_bf16x2(y0[0], y0[1]); olo.y = pack_bf16x2(y0[2], y0[3]);
        olo.z = pack_bf16x2(y0[4], y0[5]); olo.w = pack_bf16x2(y0[6], y0[7]);
        ohi.x = pack_bf16x2(y1[0], y1[1]); ohi.y = pack_bf16x2(y1[2], y1[3]);
        ohi.z = pack_bf16x2(y1[4], y1[5]); ohi.w = pack_bf16x2(y1[6], y1[7]);
    } else {
        olo.x = __float_as_uint(y0[0]); olo.y = __float_as_uint(y0[1]);
        olo.z = __float_as_uint(y0[2]); olo.w = __float_as_uint(y0[3]);
        ohi.x = __float_as_uint(y1[0]); ohi.y = __float_as_uint(y1[1]);
        ohi.z = __float_as_uint(y1[2]); ohi.w = __float_as_uint(y1[3]);
    }
    *plo = olo;
    *phi = ohi;
}

hipError_t rope_rerotate_launch(const RopeParams &p, bool bf16, hipStream_t st)
{
    if (p.n_rows == 0 || p.rot == 0) return hipSuccess;
    const int tpr = p.rot / (2 * (bf16 ? 8 : 4));
    const long threads = p.n_rows * tpr;
    const dim3 grid((unsigned)((threads + 255) / 256), (unsigned)p.Hkv);
    if (bf16) hipLaunchKernelGGL(rope_rerotate<true>, grid, dim3(256), 0, st, p);
    else hipLaunchKernelGGL(rope_rerotate<false>, grid, dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace reform

// Gathering the inputs that are recomputed (arXiv 2506.01215, Sec. 3.3 "On-Demand Cache
// Recomputation"; Alg. 1 `relevant_inputs <- GatherRelevant(input, emb)` followed by
// `model.Forward(relevant_inputs)`): out[i] = table[idx[i]] for the selected token indices.
//
// Pure streaming copy: consecutive lanes move consecutive 16-byte pieces of one row, so both the
// reads (whole rows) and the writes are fully coalesced; the number of valid indices may live in
// device memory (the union count of reform_gather_topk), so no host round trip is needed.
#include "common.h"

namespace reform {

__global__ __launch_bounds__(256) void gather_rows_kernel(RowsParams p)
{
    const long n = p.count ? min((long)*p.count, p.n_idx) : p.n_idx;
    const long total = n * p.pieces;
    const long stride = (long)gridDim.x * 256;
    for (long w = (long)blockIdx.x * 256 + threadIdx.x; w < total; w += stride) {
        const long i = w / p.pieces;
        const long piece = w - i * p.pieces;
        const long src = p.idx[i];
        if ((unsigned long)src >= (unsigned long)p.n_table) {      // never dereference a bad index
            if (p.err) atomicOr(p.err, 1);
            continue;
        }
        const v4u *s = (const v4u *)((const char *)p.table + (size_t)src * p.row_bytes) + piece;
        v4u *d = (v4u *)((char *)p.out + (size_t)i * p.row_bytes) + piece;
        *d = *s;
    }
}

hipError_t gather_rows_launch(const RowsParams &p, hipStream_t st)
{
    if (p.n_idx == 0) return hipSuccess;
    const long total = p.n_idx * p.pieces;
    const long blocks = (total + 255) / 256;
    const unsigned grid = (unsigned)(blocks < 16384 ? blocks : 16384);
    hipLaunchKernelGGL(gather_rows_kernel, dim3(grid), dim3(256), 0, st, p);
    return hipGetLastError();
}

}  // namespace reform
